"""The C-ABI library loads without a GPU, exports every symbol the header declares, and turns
every host-checkable mistake into a status code before anything is launched."""

import ctypes
import os
import re

import pytest

from paper_2605_17862_amd import binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = ctypes.c_void_p


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "fopd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fopd_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = fb.load_library()
    names = _declared_functions()
    assert set(names) == set(fb.SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    seen = set()
    for code in range(0, 10):
        s = fb.fopd_status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 10
    assert fb.fopd_status_string(99) == "unknown status"


def test_workspace_bytes():
    a = fb.fopd_workspace_bytes(512, 4)
    b = fb.fopd_workspace_bytes(147456, 64)
    assert a % 256 == 0 and b % 256 == 0 and 0 < a < b
    assert b >= 147456 * 12                      # three per-row float arrays live there
    assert fb.fopd_workspace_bytes(0, 1) >= 256


def _tok(lib, logits=4096, dt=1, T=8, V=64, ld=64, ids=4096, logp=4096, lse=4096, ws=4096, wsb=1 << 20):
    return lib.fopd_token_logprobs(P(logits), dt, T, V, ld, P(ids), None, P(logp), P(lse), None, None,
                                   P(ws), wsb, None)


def test_token_logprobs_rejects_bad_arguments_before_launch():
    lib = fb.load_library()
    assert _tok(lib, logits=None) == 1           # EINVAL
    assert _tok(lib, ids=None) == 1
    assert _tok(lib, logp=None) == 1
    assert _tok(lib, dt=2) == 4                  # EDTYPE
    assert _tok(lib, V=0) == 2                   # ESHAPE
    assert _tok(lib, T=-1) == 2
    assert _tok(lib, T=1 << 31) == 2             # one workgroup per row: the grid holds 2^31 - 1
    assert _tok(lib, ld=56) == 2
    assert _tok(lib, logits=4096 + 8) == 3       # EALIGN
    assert _tok(lib, V=60, ld=60) == 3           # bf16 pitch 120 B
    assert _tok(lib, dt=0, V=62, ld=62) == 3     # f32 pitch 248 B
    assert _tok(lib, ws=None) == 5               # EWORKSPACE
    assert _tok(lib, ws=4096 + 64) == 5
    assert _tok(lib, wsb=128) == 5


def _loss(lib, **kw):
    a = dict(logits=4096, dt=1, T=8, V=64, ld=64, ids=4096, mask=None, lb=4096, lq=4096, lqs=None,
             seq=4096, lag=4096, B=2, hp=fb.Hparams(1, 1, 0.05, 0.1), fin=None, nin=None, nroll=None, row=0,
             lse=None, lpin=None, g=1.0, loss=4096, f=None, w=None, lp=None, dl=8192, ws=4096, wsb=1 << 20)
    a.update(kw)
    return lib.fopd_loss_fwd_bwd(P(a["logits"]), a["dt"], a["T"], a["V"], a["ld"], P(a["ids"]), P(a["mask"]),
                                 P(a["lb"]), P(a["lq"]), P(a["lqs"]), P(a["seq"]), P(a["lag"]), a["B"],
                                 a["hp"], P(a["fin"]), P(a["nin"]), P(a["nroll"]), a["row"], P(a["lse"]), P(a["lpin"]),
                                 a["g"], P(a["loss"]), P(a["f"]), P(a["w"]), P(a["lp"]), P(a["dl"]),
                                 P(a["ws"]), a["wsb"], None)


def test_loss_rejects_bad_arguments_before_launch():
    lib = fb.load_library()
    assert _loss(lib, dl=None) == 1
    assert _loss(lib, loss=None) == 1
    assert _loss(lib, lb=None) == 1
    assert _loss(lib, seq=None) == 1
    assert _loss(lib, B=0) == 2
    assert _loss(lib, row=-1) == 2
    assert _loss(lib, hp=fb.Hparams(-1, 1, 0, 0)) == 1       # alpha, beta >= 0 (Eq. freshness)
    assert _loss(lib, hp=fb.Hparams(1, float("nan"), 0, 0)) == 1
    assert _loss(lib, lse=4096) == 1                          # lse_in without logp_in
    assert _loss(lib, lse=4096, lpin=4096) == 1               # ... and without freshness_in
    assert _loss(lib, row=16) == 1                            # a chunk needs scores and counts
    assert _loss(lib, fin=4096, row=16) == 1                  # ... counts still missing
    assert _loss(lib, fin=4096, nroll=4096) == 1              # roll counts only together with the sup counts
    assert _loss(lib, dl=8192 + 4) == 3
    assert _loss(lib, wsb=256) == 5


def _unit(lib, **kw):
    a = dict(logits=4096, dt=1, T=8, V=64, ld=64, ids=4096, mask=None, lb=4096, lq=4096, lqs=None,
             seq=4096, lag=4096, B=2, hp=fb.Hparams(1, 1, 0.05, 0.1), g=1.0, loss=4096, f=None, w=None, lp=None,
             rows=8192, ws=4096, wsb=1 << 20)
    a.update(kw)
    return lib.fopd_loss_fwd_bwd_unit(P(a["logits"]), a["dt"], a["T"], a["V"], a["ld"], P(a["ids"]), P(a["mask"]),
                                      P(a["lb"]), P(a["lq"]), P(a["lqs"]), P(a["seq"]), P(a["lag"]), a["B"],
                                      a["hp"], a["g"], P(a["loss"]), P(a["f"]), P(a["w"]), P(a["lp"]),
                                      P(a["rows"]), P(a["ws"]), a["wsb"], None)


def test_single_read_call_rejects_bad_arguments_before_launch():
    lib = fb.load_library()
    assert _unit(lib, logits=None) == 1
    assert _unit(lib, rows=None) == 1
    assert _unit(lib, loss=None) == 1
    assert _unit(lib, lq=None) == 1
    assert _unit(lib, lag=None) == 1
    assert _unit(lib, B=0) == 2
    assert _unit(lib, V=0) == 2
    assert _unit(lib, dt=3) == 4
    assert _unit(lib, hp=fb.Hparams(1, -2, 0, 0)) == 1
    assert _unit(lib, rows=8192 + 2) == 3
    assert _unit(lib, ws=None) == 5
    assert _unit(lib, wsb=64) == 5


def _listed(lib, **kw):
    a = dict(logits=4096, dt=1, T=8, V=64, ld=64, ids=4096, mask=None, lb=4096, lids=4096, llq=4096, k=4, floor=1e-4,
             lq=None, lqs=None, seq=4096, lag=4096, B=2, hp=fb.Hparams(1, 1, 0.05, 0.1), fin=None, nin=None,
             nroll=None, rb=0, lsein=None, lpin=None, g=1.0, loss=4096, f=None, w=None, lp=None, tl=None, dl=8192,
             ws=4096, wsb=1 << 20)
    a.update(kw)
    return lib.fopd_loss_fwd_bwd_topk_teacher(P(a["logits"]), a["dt"], a["T"], a["V"], a["ld"], P(a["ids"]),
                                              P(a["mask"]), P(a["lb"]), P(a["lids"]), P(a["llq"]), a["k"], a["floor"],
                                              P(a["lq"]), P(a["lqs"]), P(a["seq"]), P(a["lag"]), a["B"], a["hp"],
                                              P(a["fin"]), P(a["nin"]), P(a["nroll"]), a["rb"], P(a["lsein"]),
                                              P(a["lpin"]), a["g"], P(a["loss"]), P(a["f"]), P(a["w"]), P(a["lp"]),
                                              P(a["tl"]), P(a["dl"]), P(a["ws"]), a["wsb"], None)


def test_listed_teacher_call_rejects_bad_arguments_before_launch():
    lib = fb.load_library()
    assert _listed(lib, logits=None) == 1
    assert _listed(lib, dl=None) == 1
    assert _listed(lib, lids=None) == 1
    assert _listed(lib, llq=None) == 1
    assert _listed(lib, lb=None) == 1
    assert _listed(lib, loss=None) == 1
    assert _listed(lib, lqs=4096) == 1                      # the stale array without the current one
    assert _listed(lib, floor=0.0) == 1
    assert _listed(lib, floor=1.5) == 1
    assert _listed(lib, floor=float("nan")) == 1
    assert _listed(lib, hp=fb.Hparams(-1, 1, 0, 0)) == 1
    assert _listed(lib, k=0) == 2
    assert _listed(lib, k=5000) == 2
    assert _listed(lib, B=0) == 2
    assert _listed(lib, V=0) == 2
    assert _listed(lib, dt=3) == 4
    assert _listed(lib, dl=8192 + 2) == 3
    assert _listed(lib, ws=None) == 5
    need = fb.fopd_topk_workspace_bytes(8, 2, 4)
    assert need == fb.fopd_workspace_bytes(8, 2) + 2 * 256
    assert _listed(lib, wsb=need - 1) == 5
    # a chunk brings scores, counts and its slices of lse and logp; a whole batch brings none of them
    assert _listed(lib, fin=4096) == 1
    assert _listed(lib, fin=4096, nin=4096, lsein=4096) == 1
    assert _listed(lib, nin=4096) == 1
    assert _listed(lib, rb=8) == 1
    assert _listed(lib, rb=-1) == 2
    tok = lib.fopd_topk_token_loss
    assert tok(P(4096), 1, 8, 64, 64, P(4096), None, P(4096), P(4096), 4, 1e-4, P(4096), None, None) == 1
    assert tok(P(4096), 1, 8, 64, 64, P(4096), None, P(4096), P(4096), 4, 1e-4, None, P(4096), None) == 1
    assert tok(P(4096), 1, 8, 64, 64, P(4096), None, None, P(4096), 4, 1e-4, P(4096), P(4096), None) == 1
    assert tok(P(4096), 1, 8, 64, 64, P(4096), None, P(4096), P(4096), 0, 1e-4, P(4096), P(4096), None) == 2
    assert tok(P(4096), 1, 8, 64, 64, P(4096), None, P(4096), P(4096), 4, 0.0, P(4096), P(4096), None) == 1
    assert tok(P(4096 + 2), 1, 8, 64, 64, P(4096), None, P(4096), P(4096), 4, 1e-4, P(4096), P(4096), None) == 3
    assert fb.fopd_topk_workspace_bytes(163894, 64, 64) == fb.fopd_workspace_bytes(163894, 64) + 2 * 163894 * 64 * 4


def test_freshness_rejects_bad_arguments_before_launch():
    lib = fb.load_library()

    def call(logp=4096, seq=4096, lag=4096, f=4096, T=8, B=2, hp=fb.Hparams(1, 1, 0, 0), ws=4096, wsb=1 << 20):
        return lib.fopd_freshness_score(P(logp), P(4096), None, None, P(4096), None, None, P(seq), P(lag), T, B, hp,
                                        None, None, None, None, None, None, None, None, P(f), None, P(ws), wsb, None)

    assert call(logp=None) == 1
    assert call(f=None) == 1
    assert call(lag=None) == 1
    assert call(B=0) == 2
    assert call(T=-3) == 2
    assert call(hp=fb.Hparams(1, -0.5, 0, 0)) == 1
    assert call(ws=None) == 5


def test_profile_read_argument_checks():
    lib = fb.load_library()
    ms, n = ctypes.c_double(), ctypes.c_int64()
    assert lib.fopd_profile_read(8, ctypes.byref(ms), ctypes.byref(n)) == 1
    assert lib.fopd_profile_read(-1, ctypes.byref(ms), ctypes.byref(n)) == 1
    assert lib.fopd_profile_read(0, None, ctypes.byref(n)) == 1
    assert lib.fopd_profile_reset() == 0
    assert lib.fopd_profile_read(0, ctypes.byref(ms), ctypes.byref(n)) == 0 and n.value == 0


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        fb._ptr(torch.zeros(4), torch.float32, "x")


def test_set_option_checks_names_and_values():
    lib = fb.load_library()
    assert lib.fopd_set_option(b"k14_threads", 512) == 0
    assert lib.fopd_set_option(b"k14_threads", 300) == 1
    assert lib.fopd_set_option(b"k14_rows_per_cu", 2) == 0
    assert lib.fopd_set_option(b"k14_rows_per_cu", 0) == 1
    assert lib.fopd_set_option(b"k14_regs_grid", 512) == 0
    assert lib.fopd_set_option(b"k14_regs_grid", -1) == 1
    assert lib.fopd_set_option(b"k14_regs_grid", 5000) == 1
    assert lib.fopd_set_option(b"k4_regs", 0) == 0
    assert lib.fopd_set_option(b"k4_regs", 2) == 1
    assert lib.fopd_set_option(b"k4_regs", 1) == 0
    assert lib.fopd_set_option(b"lm_head_compact", 0) == 0
    assert lib.fopd_set_option(b"lm_head_compact", 2) == 1
    assert lib.fopd_set_option(b"lm_head_compact", 1) == 0
    assert lib.fopd_set_option(b"no_such_option", 1) == 1
    assert lib.fopd_set_option(None, 1) == 1
    # back to the defaults: the options are process-wide
    assert lib.fopd_set_option(b"k14_threads", 256) == 0
    assert lib.fopd_set_option(b"k14_rows_per_cu", 6) == 0
    assert lib.fopd_set_option(b"k14_regs_grid", 0) == 0


def test_header_is_plain_c(tmp_path):
    """include/fopd.h must compile as C99 (no C++ in the boundary) and declare what the library exports."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("gcc not available")
    src = tmp_path / "use_fopd.c"
    src.write_text('#include "fopd.h"\n'
                   "int main(void) {\n"
                   "  fopd_hparams hp = {1.0f, 1.0f, 0.05f, 0.1f};\n"
                   "  fopd_refresh_config rc = {0.3f, 0.5f, 0.5f, 200};\n"
                   "  fopd_refresh_state rs = {-1, 0};\n"
                   "  float agg[3] = {0.1f, 1.0f, 1.0f};\n"
                   "  (void)hp; (void)fopd_status_string(FOPD_OK);\n"
                   "  (void)fopd_workspace_bytes(16, 2);\n"
                   "  return fopd_refresh_decide(agg, &rc, &rs, 0, 0) == 1 ? 0 : 1;\n"
                   "}\n")
    obj = tmp_path / "use_fopd.o"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                        "-c", str(src), "-o", str(obj)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def _lmh(lib, hidden=4096, ldh=64, weight=8192, ldw=64, T=8, V=100, d=64, ids=4096, logp=4096, lse=4096, ws=4096,
         wsb=1 << 20):
    return lib.fopd_lm_head_token_logprobs(P(hidden), ldh, P(weight), ldw, T, V, d, P(ids), None, P(logp), P(lse),
                                           P(ws), wsb, None)


def test_projection_entry_point_rejects_bad_arguments_before_launch():
    lib = fb.load_library()
    assert _lmh(lib, hidden=None) == 1           # EINVAL
    assert _lmh(lib, weight=None) == 1
    assert _lmh(lib, ids=None) == 1
    assert _lmh(lib, lse=None) == 1
    assert _lmh(lib, d=0) == 2                   # ESHAPE
    assert _lmh(lib, d=96, ldh=96, ldw=96) == 2  # hidden size must be a multiple of 64
    assert _lmh(lib, ldh=32) == 2                # pitch below d
    assert _lmh(lib, ldw=56) == 2
    assert _lmh(lib, T=-1) == 2
    assert _lmh(lib, V=0) == 2
    assert _lmh(lib, T=1 << 20, ldh=1 << 11) == 5           # T * ldh reaches 2^31: row blocks; the workspace is too small
    assert _lmh(lib, T=1 << 20, ldh=1 << 11, hidden=4104, wsb=1 << 30) == 3
    assert _lmh(lib, V=1 << 19, ldw=1 << 12) == 2           # V * ldw reaches 2^31
    assert _lmh(lib, hidden=4104) == 3           # EALIGN: base not on 16 bytes
    assert _lmh(lib, ldh=68) == 3                # row pitch not a multiple of 16 bytes
    assert _lmh(lib, ws=None) == 5               # EWORKSPACE
    assert _lmh(lib, ws=4100) == 5
    assert _lmh(lib, wsb=1024) == 5
    assert _lmh(lib, T=0) == 0                   # nothing to do, nothing launched


def _lml(lib, **kw):
    a = dict(hidden=4096, ldh=64, weight=4096, ldw=64, T=128, V=100, d=64, ids=4096, lb=4096, lq=4096, seq=4096, lag=4096,
             B=2, hp=fb.Hparams(1, 1, 0.05, 0.1), fin=4096, nin=None, nroll=None, host=None, chunk=64, loss=4096,
             f=None, w=None, lp=4096, lse=4096, dh=8192, dw=8192, ws=4096, wsb=1 << 24)
    a.update(kw)
    host = a["host"]
    keep = (ctypes.c_int32 * len(host))(*host) if host is not None else None
    return lib.fopd_lm_head_loss_fwd_bwd(P(a["hidden"]), a["ldh"], P(a["weight"]), a["ldw"], a["T"], a["V"], a["d"],
                                         P(a["ids"]), None, P(a["lb"]), P(a["lq"]), P(a["seq"]), P(a["lag"]), a["B"],
                                         a["hp"], P(a["fin"]), P(a["nin"]), P(a["nroll"]),
                                         None if keep is None else ctypes.cast(keep, ctypes.c_void_p), 1.0, a["chunk"],
                                         P(a["loss"]), P(a["f"]), P(a["w"]), P(a["lp"]), P(a["lse"]), P(a["dh"]), 64,
                                         P(a["dw"]), 64, 0, P(a["ws"]), a["wsb"], None)


def test_projection_loss_rejects_bad_arguments_before_launch():
    lib = fb.load_library()
    assert _lml(lib, hidden=None) == 1
    assert _lml(lib, dh=None) == 1                                # a weight gradient without the hidden one
    assert _lml(lib, chunk=32) == 2                               # rows per chunk: a multiple of 64
    assert _lml(lib, d=96, ldh=96, ldw=96) == 2
    assert _lml(lib, nroll=4096) == 1                             # roll counts only together with the sup counts
    assert _lml(lib, hp=fb.Hparams(-1, 1, 0, 0)) == 1
    assert _lml(lib, wsb=4096) == 5
    # scores formed inside the call: the host needs the lengths, whole samples per chunk, lengths adding up to T
    assert _lml(lib, fin=None) == 1
    assert _lml(lib, fin=None, host=[64, 64], nin=4096) == 1
    assert _lml(lib, fin=None, host=[64, 32]) == 2                # 96 rows, T = 128
    assert _lml(lib, fin=None, host=[-1, 129]) == 2


def test_projection_workspace_bytes():
    a = fb.fopd_lm_head_workspace_bytes(1)
    b = fb.fopd_lm_head_workspace_bytes(256)
    c = fb.fopd_lm_head_workspace_bytes(257)
    # the strip pairs are padded to whole 256-token tiles; the row map and the prefix counts take 8 bytes a row
    assert a <= b < c and b - a <= 8 * 255 + 512 and a % 256 == 0 and c - b >= 32 * 256 * 8
    assert fb.fopd_lm_head_workspace_bytes(163894) >= 163894 * 32 * 8
    assert fb.fopd_lm_head_workspace_bytes(0) >= 256


def _lml_listed(lib, **kw):
    a = dict(hidden=4096, ldh=64, weight=4096, ldw=64, T=128, V=100, d=64, ids=4096, lb=4096, lids=4096, llq=4096, k=4,
             floor=1e-4, lq=None, lqs=None, seq=4096, lag=4096, B=2, hp=fb.Hparams(1, 1, 0.05, 0.1), host=[64, 64],
             chunk=64, loss=4096, lp=4096, lse=4096, dh=8192, dw=8192, ws=4096, wsb=1 << 24, fin=None, nin=None,
             nroll=None)
    a.update(kw)
    host = a["host"]
    keep = (ctypes.c_int32 * len(host))(*host) if host is not None else None
    return lib.fopd_lm_head_loss_fwd_bwd_topk_teacher(
        P(a["hidden"]), a["ldh"], P(a["weight"]), a["ldw"], a["T"], a["V"], a["d"], P(a["ids"]), None, P(a["lb"]),
        P(a["lids"]), P(a["llq"]), a["k"], a["floor"], P(a["lq"]), P(a["lqs"]), P(a["seq"]), P(a["lag"]), a["B"], a["hp"],
        P(a["fin"]), P(a["nin"]), P(a["nroll"]),
        None if keep is None else ctypes.cast(keep, ctypes.c_void_p), 1.0, a["chunk"], P(a["loss"]), None, None,
        P(a["lp"]), P(a["lse"]), None, P(a["dh"]), 64, P(a["dw"]), 64, 0, P(a["ws"]), a["wsb"], None)


def test_projection_loss_with_listed_teacher_rejects_bad_arguments_before_launch():
    lib = fb.load_library()
    assert _lml_listed(lib, hidden=None) == 1
    assert _lml_listed(lib, lids=None) == 1
    assert _lml_listed(lib, llq=None) == 1
    assert _lml_listed(lib, host=None) == 1                       # whole samples per chunk: the host needs the lengths
    assert _lml_listed(lib, nin=4096) == 1                        # counts without scores
    assert _lml_listed(lib, fin=4096, nroll=4096) == 1            # roll counts only together with the sup counts
    assert _lml_listed(lib, fin=4096, dh=None, dw=None) == 1      # scoring with scores supplied
    assert _lml_listed(lib, lqs=4096) == 1                        # the stale array without the current one
    assert _lml_listed(lib, floor=0.0) == 1
    assert _lml_listed(lib, k=0) == 2
    assert _lml_listed(lib, k=4097) == 2
    assert _lml_listed(lib, chunk=32) == 2
    assert _lml_listed(lib, host=[100, 27]) == 2                  # lengths that do not add up to T
    assert _lml_listed(lib, wsb=4096) == 5
    plain = fb.fopd_lm_head_loss_workspace_bytes(128, 100, 64, 2, 64)
    listed = fb.fopd_lm_head_loss_topk_workspace_bytes(128, 100, 64, 2, 64, 4)
    assert listed > plain and listed - plain < 128 * 4 + 64 * 4 * (3 + 4 * 4) + 8 * 256 + 1
    assert _lml_listed(lib, wsb=listed - 1) == 5
