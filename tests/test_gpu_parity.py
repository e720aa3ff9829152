"""GPU parity: the HIP library, called through its C ABI, against the float64 oracle on the same
seeded inputs.  Every test here needs an MI355X (`-m gpu`)."""

import numpy as np
import pytest
import torch

from oracle import fopd_oracle as orc
from paper_2605_17862_amd import binding as fb
from harness import workloads as wl
from paper_2605_17862_amd.loss_pass import DEFAULT_HPARAMS, LossPass
from parity_util import (KL_ROW_ATOL, assert_close, check_grad_rows, check_grad_rows_full_kl, coef_uncertainty,
                         floor_report, np64, oracle_full)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HP = DEFAULT_HPARAMS


def _say(msg):
    print("[gpu-parity] " + msg, flush=True)


@pytest.fixture(autouse=True)
def _dlogits_floor_accounting(request):
    """After each test: how many gradient elements needed more than the plain 2-ulp bound, and why."""
    floor_report()
    yield
    st, line = floor_report()
    if st["elements"]:
        _say("%s: %s" % (request.node.name, line))


def _pass_for(w, alloc_dlogits=True):
    return LossPass(w["T"], w["V"], w["B"], w["dtype"], ld=w["ld"], device=DEV, alloc_dlogits=alloc_dlogits)


def _sync_ok(lp):
    st, flags = lp.status()
    assert st == 0 and flags == 0, "device flags %d (%s)" % (flags, fb.fopd_status_string(st))


def _compare_everything(w, hp, grad_scale=1.0, staged=True):
    """Fused call (and optionally the staged calls) against the oracle on a small workload."""
    ref = oracle_full(w, hp, grad_scale)
    lp = _pass_for(w)
    lp.loss_fwd_bwd(w, hp, grad_scale)
    _sync_ok(lp)
    live = np64(w["mask"]) != 0
    assert_close("logp", np64(lp.logp), ref["logp"], atol=1e-4)
    # the fp32 log-prob keeps relative accuracy as p_y -> 1
    assert_close("logp (relative)", np64(lp.logp)[live], ref["logp"][live], rtol=1e-5, atol=2e-6)
    assert_close("freshness", np64(lp.freshness), ref["freshness"], rtol=1e-5)
    assert_close("weights", np64(lp.weights), ref["weights"], atol=1e-5 * ref["freshness"] + 1e-12)
    assert abs(float(lp.loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-12, (float(lp.loss), ref["loss"])
    eps_c = coef_uncertainty(ref, hp, grad_scale, w["B"], np64(w["mask"]))
    V = w["V"]
    got = np64(lp.dlogits)
    check_grad_rows(got[:, :V], np64(w["logits"])[:, :V], ref["gather_idx"] - np.arange(w["T"]) * w["ld"],
                    ref["lse"], ref["coef"], eps_c, w["dtype"])
    # samples the oracle gates by a clear margin must have bit-exact zero rows
    cu = ref["cu_seqlens"]
    for i in range(w["B"]):
        if min(ref["n_train"][i], ref["n_roll"][i]) == 0 or ref["freshness"][i] < hp[2] * (1 - 1e-4):
            assert not np.any(got[cu[i]:cu[i + 1], :V]), "gated/invalid sample %d has non-zero rows" % i
            assert float(lp.weights[i]) == 0.0
    if staged:
        st = _pass_for(w, alloc_dlogits=False)
        st.token_logprobs(w, want_entropy=True)
        st.freshness_score(w, hp)
        _sync_ok(st)
        # token entropy comes out of the same pass and must not disturb the log-probs
        H = orc.token_entropy(np64(w["logits"])[:, :w["V"]], np64(w["mask"]))
        assert_close("entropy", np64(st.entropy), H, rtol=2e-5, atol=2e-5)
        assert np.array_equal(np64(st.gather_idx), ref["gather_idx"]) and st.gather_idx.dtype == torch.int64
        assert np.array_equal(np64(st.cu_seqlens), ref["cu_seqlens"]) and st.cu_seqlens.dtype == torch.int64
        assert np.array_equal(np64(st.n_train), ref["n_train"]) and st.n_train.dtype == torch.int32
        assert np.array_equal(np64(st.n_roll), ref["n_roll"]) and st.n_roll.dtype == torch.int32
        assert torch.equal(st.logp, lp.logp)                         # same kernel, same bits
        assert_close("lse", np64(st.lse), ref["lse"],
                     atol=1e-4 + np.spacing(np.abs(ref["lse"]).astype(np.float32)).astype(np.float64))
        assert_close("D_roll", np64(st.D_roll), ref["D_roll"], rtol=2e-5, atol=1e-9)
        assert_close("D_sup", np64(st.D_sup), ref["D_sup"], rtol=2e-5, atol=1e-9)
        # a mean of fp32-rounded log-probs (each within 1e-6 of the exact one): absolute, not relative
        assert_close("ell", np64(st.ell), ref["ell"], rtol=2e-5, atol=1e-6)
        assert_close("cover", np64(st.cover), ref["cover"], rtol=1e-6)
        assert_close("cover_roll", np64(st.cover_roll), ref["cover_roll"], rtol=1e-6)
        assert_close("freshness (staged)", np64(st.freshness), ref["freshness"], rtol=1e-5)
        assert torch.equal(st.freshness, lp.freshness)
        assert_close("agg", np64(st.agg), ref["agg"], rtol=1e-5)
    return ref, lp


# ---------------------------------------------------------------------------------------
# the paper-shaped workloads
# ---------------------------------------------------------------------------------------

def test_tiny_config_all_outputs():
    _say("tiny: T=512 V=4096 f32 seed 0")
    w = wl.generate("tiny", DEV, seed=0)
    ref, lp = _compare_everything(w, HP)
    assert np.all(ref["weights"] > 0)                 # tiny never gates
    # lag-0 sample: behaviour log-probs equal the current ones up to fp32 -> ratio 1, fresh score
    assert abs(float(lp.freshness[0]) - 1.0) < 1e-4
    # lag-only special case (alpha = beta = 0): f = 1 / (tau + 1) exactly
    lp2 = _pass_for(w)
    lp2.loss_fwd_bwd(w, (0.0, 0.0, 0.05, 0.1))
    assert np.array_equal(np64(lp2.freshness), (1.0 / (np64(w["lag"]) + 1.0)).astype(np.float32).astype(np.float64))


REPLICAS = {
    "reasoning": dict(B=6, len_lo=20, len_hi=48),
    "tooluse": dict(B=3, turns=3, obs_lo=3, obs_hi=8, resp_lo=6, resp_hi=20),
    "coding": dict(B=2, total_len=96, resp_lo=8, resp_hi=24, obs_lo=4, obs_hi=12),
    "largevocab": dict(B=4, len_lo=16, len_hi=16),
}


@pytest.mark.parametrize("name", sorted(REPLICAS))
def test_reduced_replica_at_full_vocabulary(name):
    _say("replica %s at full V, seed 3" % name)
    w = wl.generate(name, DEV, seed=3, row_block=64, **REPLICAS[name])
    ref, _ = _compare_everything(w, HP, grad_scale=1.0)
    if name == "coding":
        assert np.all(ref["D_sup"][ref["n_train"] > 0] >= 0) and np.any(ref["D_sup"] > 0)
    if name == "largevocab":
        assert np.any(ref["weights"] == 0) and np.any(ref["weights"] > 0)    # both gate branches


# ---------------------------------------------------------------------------------------
# shapes: ragged tails, tiny vocabularies, padding, empty and masked samples
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype,V,ld", [("bf16", 5003, 5008), ("bf16", 100, 104), ("bf16", 8, 8), ("bf16", 7, 8),
                                        ("bf16", 1, 8), ("bf16", 9001, 9008), ("bf16", 8200, 8200),
                                        ("f32", 5003, 5004), ("f32", 3, 4), ("f32", 4097, 4100)])
def test_ragged_vocabulary_and_padding(dtype, V, ld):
    _say("ragged V=%d ld=%d %s" % (V, ld, dtype))
    w = wl.generate("reasoning", DEV, seed=5, B=5, len_lo=3, len_hi=9, V=V, ld=ld, dtype=dtype,
                    boost=min(4, V))
    w["logits"][:, V:] = 123.0                         # padding columns must be ignored ...
    lp = _pass_for(w)
    lp.dlogits.fill_(-7.0)
    _compare_everything(w, HP, grad_scale=3.0)
    lp.loss_fwd_bwd(w, HP, 3.0)
    torch.cuda.synchronize()
    if ld > V:                                         # ... and never written
        assert bool((lp.dlogits[:, V:] == -7.0).all())


def test_random_shapes_sweep():
    """Forty seeded random problems: vocabulary size, padding, storage type, sample count and lengths,
    masks (one or two aligned sets), empty samples, lags (some gated), hyper-parameters and upstream scale
    all vary."""
    rs = np.random.RandomState(77)
    for case in range(40):
        dtype = "bf16" if rs.rand() < 0.7 else "f32"
        per = 8 if dtype == "bf16" else 4
        V = int(rs.choice([1, 2, 5, 8, 9, 31, 64, 255, 1000, 2049, 4096, 10007, 32768, 65537]))
        ld = ((V + per - 1) // per) * per + per * int(rs.randint(0, 3))
        B = int(rs.randint(1, 7))
        hp = (float(rs.choice([0.0, 0.5, 1.0, 2.0])), float(rs.choice([0.0, 1.0])),
              float(rs.choice([0.0, 0.05, 0.2])), float(rs.choice([0.0, 0.1, 1.0])))
        g = float(rs.choice([1.0, 0.125, -2.0]))
        _say("random case %d: %s V=%d ld=%d B=%d hp=%s g=%g" % (case, dtype, V, ld, B, hp, g))
        # every third problem keeps the two aligned sets apart (mask bytes 2 and 3 among the kept rows)
        split = dict(aligned_split=(0.3, 0.3)) if case % 3 == 2 else {}
        w = wl.generate("tooluse", DEV, seed=1000 + case, B=B, turns=int(rs.randint(1, 4)), obs_lo=0,
                        obs_hi=int(rs.randint(0, 5)), resp_lo=0, resp_hi=int(rs.randint(1, 9)), V=V, ld=ld,
                        dtype=dtype, boost=min(3, V), lag_lo=0, lag_hi=int(rs.choice([0, 3, 25])),
                        stale_sigma=float(rs.choice([0.0, 0.1])), row_block=64, **split)
        if w["T"] == 0:
            continue
        _compare_everything(w, hp, grad_scale=g, staged=True)


def test_empty_masked_and_gated_samples():
    _say("empty / fully masked / gated samples")
    w = wl.generate("reasoning", DEV, seed=6, B=6, len_lo=5, len_hi=12, V=2048)
    seq = w["seq_lens_host"].copy()
    T = w["T"]
    # sample 1 becomes empty (its rows go to sample 2), sample 3 is fully masked, sample 5 is very stale
    seq[2] += seq[1]
    seq[1] = 0
    cu = np.concatenate([[0], np.cumsum(seq)])
    mask = np.ones(T, dtype=np.uint8)
    mask[cu[3]:cu[4]] = 0
    mask[cu[0] + 1] = 0
    lag = w["lag_host"].copy()
    lag[5] = 60
    w["seq_lens"] = torch.from_numpy(seq).to(DEV)
    w["mask"] = torch.from_numpy(mask).to(DEV)
    w["lag"] = torch.from_numpy(lag).to(DEV)
    ref, lp = _compare_everything(w, HP)
    assert ref["n_train"][1] == 0 and ref["n_train"][3] == 0
    assert float(lp.freshness[1]) == 0.0 and float(lp.freshness[3]) == 0.0
    assert float(lp.weights[5]) == 0.0 and float(lp.freshness[5]) > 0.0
    assert float(lp.logp[cu[0] + 1]) == 0.0
    # a negative gate threshold must not revive invalid samples
    lp.loss_fwd_bwd(w, (1.0, 1.0, -0.5, 0.1))
    torch.cuda.synchronize()
    assert float(lp.weights[1]) == 0.0 and float(lp.weights[3]) == 0.0 and float(lp.weights[5]) > 0.5


def test_zero_rows_is_a_valid_call():
    """T = 0 (an empty chunk): nothing is read or written except loss = 0 and the per-sample outputs."""
    B = 3
    dummy = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    f32 = torch.zeros(8, device=DEV)
    i32 = torch.zeros(8, dtype=torch.int32, device=DEV)
    lp = LossPass(1, 64, B, "bf16", device=DEV)
    lp.loss.fill_(7.0)
    fb.fopd_loss_fwd_bwd(dummy, lp.dt, 0, 64, 64, i32, None, f32, f32, None, i32[:B], i32[:B], B, HP, None, None, None, 0,
                         None, None, 1.0, lp.loss, lp.freshness, lp.weights, None, dummy, lp.workspace)
    _sync_ok(lp)
    assert float(lp.loss) == 0.0 and not bool(lp.freshness.any()) and not bool(lp.weights.any())
    fb.fopd_token_logprobs(dummy, lp.dt, 0, 64, 64, i32, None, f32, f32, None, None, lp.workspace)
    fb.fopd_freshness_score(f32, f32, None, None, f32, None, None, i32[:B], i32[:B], 0, B, HP, lp.cu_seqlens, lp.n_train,
                            None, None, None, None, lp.cover, None, lp.freshness, lp.agg, lp.workspace)
    _sync_ok(lp)
    assert not bool(lp.cu_seqlens.any()) and not bool(lp.n_train.any()) and not bool(lp.agg.any())


def test_all_rows_masked_gives_zero_everything():
    w = wl.generate("reasoning", DEV, seed=7, B=3, len_lo=4, len_hi=6, V=1024)
    w["mask"].zero_()
    lp = _pass_for(w)
    lp.dlogits.fill_(1.0)
    lp.loss_fwd_bwd(w, HP)
    _sync_ok(lp)
    assert float(lp.loss) == 0.0 and not bool(lp.dlogits.any()) and not bool(lp.freshness.any())
    lp.token_logprobs(w)
    lp.freshness_score(w, HP)
    _sync_ok(lp)
    assert not bool(lp.n_train.any()) and not bool(lp.cover.any()) and float(lp.agg[0]) == 0.0


def test_in_place_gradient_and_determinism():
    _say("in-place dlogits and run-to-run determinism")
    w = wl.generate("reasoning", DEV, seed=8, B=8, len_lo=20, len_hi=40, V=151936, row_block=64)
    lp = _pass_for(w)
    lp.loss_fwd_bwd(w, HP)
    first = lp.dlogits.clone()
    loss1, f1 = lp.loss.clone(), lp.freshness.clone()
    lp.dlogits.zero_()
    lp.loss_fwd_bwd(w, HP)
    torch.cuda.synchronize()
    assert torch.equal(first, lp.dlogits) and torch.equal(loss1, lp.loss) and torch.equal(f1, lp.freshness)
    z = w["logits"].clone()
    lp.loss_fwd_bwd(dict(w, logits=z), HP, dlogits=z)          # dlogits aliases logits
    _sync_ok(lp)
    assert torch.equal(first, z)


# ---------------------------------------------------------------------------------------
# numerics at the extremes
# ---------------------------------------------------------------------------------------

def test_extreme_rows():
    _say("extreme rows: p_y -> 1, p_y -> 0, -inf entries, +-8000 magnitudes")
    V, T = 4096, 6
    g = torch.Generator().manual_seed(9)
    z = torch.randn(T, V, generator=g) * 2.0
    y = torch.tensor([5, 17, 100, 9, 4095, 0], dtype=torch.int32)
    z[0, 5] = 60.0                         # p_y = 1 - 4e-23
    z[1, 17] = 24.0                        # p_y = 1 - 1e-6
    z[2, 100] = -80.0                      # p_y ~ 1e-39 relative to the rest
    z[3, 100:200] = float("-inf")          # masked-out vocabulary entries
    z[4] *= 2000.0                         # logits of magnitude up to ~ 8000
    z[5, :] = 3.0                          # constant row: lp = -log V
    zb = z.to(torch.bfloat16)
    seq = torch.tensor([T], dtype=torch.int32)
    w = dict(T=T, V=V, ld=V, B=1, dtype="bf16", logits=zb.to(DEV), token_ids=y.to(DEV),
             mask=torch.ones(T, dtype=torch.uint8, device=DEV),
             behav_logp=torch.full((T,), -0.5, device=DEV), teacher_logp=torch.full((T,), -0.4, device=DEV),
             teacher_logp_stale=None, seq_lens=seq.to(DEV), lag=torch.zeros(1, dtype=torch.int32, device=DEV))
    lp = _pass_for(w)
    lp.token_logprobs(w)
    _sync_ok(lp)
    lse_ref, lp_ref = orc.token_logprobs(np64(zb), y.numpy(), None)
    got = np64(lp.logp)
    assert np.all(np.isfinite(got))
    # rows 0, 1: z_y - lse cancels in float64 too; -log1p(sum_{v != y} exp(z_v - z_y)) is the accurate form
    for r in (0, 1):
        zz = np64(zb[r])
        others = np.delete(zz, int(y[r]))
        lp_ref[r] = -np.log1p(np.sum(np.exp(others - zz[int(y[r])])))
    assert_close("logp extreme", got, lp_ref, rtol=1e-5, atol=1e-40)
    assert_close("lse extreme", np64(lp.lse), lse_ref, rtol=1e-6, atol=1e-5)
    assert abs(got[5] + np.log(V)) < 1e-6
    lp.token_logprobs(w, want_entropy=True)
    _sync_ok(lp)
    assert np.array_equal(np64(lp.logp), got)                       # same log-probs with the entropy variant
    H = orc.token_entropy(np64(zb), None)
    # the oracle's log p_y = z_y - lse cancels in float64 when p_y -> 1 (row 0 loses its p_y log p_y term)
    assert_close("entropy extreme", np64(lp.entropy), H, rtol=2e-5, atol=8 * np.spacing(np.abs(lse_ref)))
    assert abs(float(lp.entropy[5]) - np.log(V)) < 1e-5 and float(lp.entropy[0]) < 1e-18
    # gradient of the same rows: the sampled-token entry is c * (p_y - 1), accurate as p_y -> 1
    ref = oracle_full(w, (1.0, 1.0, 0.0, 0.1))
    lp.loss_fwd_bwd(w, (1.0, 1.0, 0.0, 0.1))
    _sync_ok(lp)
    gg = np64(lp.dlogits)
    c1 = ref["coef"][1]
    want = c1 * np.expm1(lp_ref[1])
    assert abs(gg[1, 17] - want) <= 2 * orc.bf16_ulp(want) + abs(want) * 1e-4
    assert np.all(np.isfinite(gg)) and np.all(gg[3, 100:200] == 0.0)
    # a sampled token whose logit is -inf (probability 0): lp = -inf, lse finite and equal to the oracle's;
    # and a row whose only finite logit is the sampled one: lp = 0, lse = z_y
    z2 = zb.clone()
    z2[2, 100] = float("-inf")
    z2[5, :] = float("-inf")
    z2[5, 0] = 1.5
    w2 = dict(w, logits=z2.to(DEV))
    lp.token_logprobs(w2)
    _sync_ok(lp)
    lse2, lp2 = orc.token_logprobs(np64(z2), y.numpy(), None)
    assert float(lp.logp[2]) == float("-inf") and lp2[2] == float("-inf")
    assert abs(float(lp.lse[2]) - lse2[2]) <= 1e-5 and np.isfinite(float(lp.lse[2]))
    assert float(lp.logp[5]) == 0.0 and float(lp.lse[5]) == 1.5


# ---------------------------------------------------------------------------------------
# modes of fopd_loss_fwd_bwd
# ---------------------------------------------------------------------------------------

def _scored_reference(w, hp, f_used, n_used, grad_scale=1.0):
    """Oracle gradient when the scores are given: weights from f_used, everything else as usual."""
    V = w["V"]
    z = np64(w["logits"])[:, :V]
    y, mask = np64(w["token_ids"]), np64(w["mask"])
    lse, lp = orc.token_logprobs(z, y, mask)
    delta, rho, adv, k_roll, _ = orc.token_terms(lp, np64(w["behav_logp"]), np64(w["teacher_logp"]), None)
    cu = orc.segment_offsets(np64(w["seq_lens"]))
    wts = orc.freshness_weights(f_used, hp[2], n_used)
    coef = orc.grad_coefficients(delta, rho, adv, mask, cu, n_used, wts, hp[3], grad_scale)
    B = w["B"]
    per_tok = np.zeros(w["T"])
    for i in range(B):
        for t in range(int(cu[i]), int(cu[i + 1])):
            if mask[t] and n_used[i] > 0:
                per_tok[t] = wts[i] / (B * int(n_used[i])) * ((lp[t] - np64(w["teacher_logp"])[t]) + hp[3] * k_roll[t])
    ref = dict(cu_seqlens=cu, n_train=n_used, freshness=np.asarray(f_used, dtype=np.float64), weights=wts,
               coef=coef, adv=adv, rho=rho, delta=delta, lse=lse, logp=lp, loss_terms=per_tok)
    return ref, z, y


def test_scores_supplied_and_chunked_flow():
    _say("freshness_in mode and the chunked flow (chunks cut samples)")
    w = wl.generate("coding", DEV, seed=11, B=3, total_len=64, resp_lo=6, resp_hi=16, obs_lo=3, obs_hi=9,
                    V=151936, row_block=64)
    T, V, B = w["T"], w["V"], w["B"]
    hp = (1.0, 1.0, 0.05, 0.3)
    full = _pass_for(w)
    # phase 1 of the chunked flow: log-probs chunk by chunk (chunk = 40 rows, samples are 64 rows)
    chunk = 40
    for a in range(0, T, chunk):
        full.token_logprobs(w, rows=(a, min(a + chunk, T)))
    full.freshness_score(w, hp)
    _sync_ok(full)
    f_gpu, n_gpu = full.freshness.clone(), full.n_train.clone()

    # (a) scores supplied, whole samples, counts taken from the mask
    sc = _pass_for(w)
    fb.fopd_loss_fwd_bwd(w["logits"], sc.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                         w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp,
                         f_gpu, None, None, 0, None, None, 2.0, sc.loss, sc.freshness, sc.weights, sc.logp,
                         sc.dlogits, sc.workspace)
    _sync_ok(sc)
    assert torch.equal(sc.freshness, f_gpu)
    ref, z, y = _scored_reference(w, hp, np64(f_gpu), np64(n_gpu), 2.0)
    eps_c = coef_uncertainty(ref, hp, 2.0, B, np64(w["mask"]))
    check_grad_rows(np64(sc.dlogits)[:, :V], z, y, ref["lse"], ref["coef"], eps_c, "bf16")
    L = float(np.sum(ref["loss_terms"]))
    assert abs(float(sc.loss) - L) <= 1e-5 * abs(L)
    assert_close("weights (scored)", np64(sc.weights), ref["weights"], rtol=1e-6, atol=1e-9)

    # (b) phase 3 of the chunked flow: gradient chunk by chunk from stored lse / logp
    ck = _pass_for(w)
    ck.dlogits.fill_(9.0)
    parts = []
    for a in range(0, T, chunk):
        b = min(a + chunk, T)
        part = torch.zeros(1, device=DEV)
        stale = w["teacher_logp_stale"]
        fb.fopd_loss_fwd_bwd(w["logits"][a:b], ck.dt, b - a, V, w["ld"], w["token_ids"][a:b], w["mask"][a:b],
                             w["behav_logp"][a:b], w["teacher_logp"][a:b], None if stale is None else stale[a:b],
                             w["seq_lens"], w["lag"], B, hp, f_gpu, n_gpu, None, a, full.lse[a:b], full.logp[a:b],
                             2.0, part, None, ck.weights, None, ck.dlogits[a:b], ck.workspace)
        parts.append(part)
    _sync_ok(ck)
    # (a) held each row in registers (1024 lanes), the log-probs of (b) come from the 256-lane pass: the two sum
    # a row in different orders, so entries may differ by one unit of the storage type
    xd, yd = np64(ck.dlogits), np64(sc.dlogits)
    assert bool(np.all(np.abs(xd - yd) <= orc.bf16_ulp(yd))) and float(np.mean(xd == yd)) > 0.99
    tot = sum(float(p) for p in parts)
    assert abs(tot - float(sc.loss)) <= 2e-6 * abs(float(sc.loss))
    assert torch.equal(ck.weights, sc.weights)
    # with the register path switched off the one-kernel call uses the 256-lane partition: the same bits
    try:
        fb.fopd_set_option("k14_regs", 0)
        sc0 = _pass_for(w)
        fb.fopd_loss_fwd_bwd(w["logits"], sc0.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                             w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp,
                             f_gpu, None, None, 0, None, None, 2.0, sc0.loss, sc0.freshness, sc0.weights, sc0.logp,
                             sc0.dlogits, sc0.workspace)
        _sync_ok(sc0)
        assert torch.equal(ck.dlogits, sc0.dlogits) and torch.equal(sc0.logp, full.logp)
    finally:
        fb.fopd_set_option("k14_regs", 1)


@pytest.mark.parametrize("threads,rows_per_cu,dtype,V,ld", [(256, 6, "bf16", 5003, 5008), (512, 2, "bf16", 40000, 40000),
                                                          (1024, 1, "bf16", 151936, 151936), (256, 8, "f32", 4097, 4100),
                                                          (1024, 2, "f32", 3, 4), (512, 4, "bf16", 1, 8),
                                                          (0, 6, "bf16", 151936, 151936), (0, 6, "bf16", 155648, 155648),
                                                          (0, 6, "bf16", 16392, 16392), (0, 6, "f32", 20003, 20004),
                                                          (0, 6, "bf16", 155656, 155656)])
def test_two_passes_per_row_kernel_matches_separate_kernels(threads, rows_per_cu, dtype, V, ld):
    """With scores supplied and no stored log-probs, one kernel makes both passes over each row.  With
    256 lanes per row (the default, and the partition the log-prob kernel uses) it must give the bits
    of the separate log-prob, coefficient and gradient kernels; other lane counts sum the row in a
    different order, so they may differ by one unit in the last place.  Covered: masks, gated samples,
    padding, a row offset and an aliased output."""
    _say("two-pass-per-row kernel: %d lanes, %d rows/CU, %s V=%d" % (threads, rows_per_cu, dtype, V))
    w = wl.generate("tooluse", DEV, seed=13, B=5, turns=2, obs_lo=2, obs_hi=5, resp_lo=3, resp_hi=9, V=V, ld=ld,
                    dtype=dtype, boost=min(4, V), lag_lo=0, lag_hi=30, row_block=32)
    T, B = w["T"], w["B"]
    hp = (1.0, 1.0, 0.05, 0.3)
    st = _pass_for(w)
    st.token_logprobs(w)
    st.freshness_score(w, hp)
    _sync_ok(st)
    f_gpu, n_gpu = st.freshness.clone(), st.n_train.clone()
    assert bool((f_gpu < 0.05).any()) and bool((f_gpu > 0.05).any())        # gated and live samples

    def call(lp, a, b, lse, logp_in, logp_out, out, n_in):
        fb.fopd_loss_fwd_bwd(w["logits"][a:b], lp.dt, b - a, V, ld, w["token_ids"][a:b], w["mask"][a:b],
                             w["behav_logp"][a:b], w["teacher_logp"][a:b], None, w["seq_lens"], w["lag"], B, hp,
                             f_gpu, n_in, None, a, lse, logp_in, 0.5, lp.loss, None, lp.weights, logp_out, out,
                             lp.workspace)

    ref = _pass_for(w)                    # separate kernels: stored lse / logp, gradient kernel only
    ref.dlogits.fill_(3.0)
    call(ref, 0, T, st.lse, st.logp, None, ref.dlogits, n_gpu)
    _sync_ok(ref)
    try:
        # threads == 0: the default setting, rows held in registers when they fit (1024 lanes; the longest row
        # that fits has 19456 vectors, V = 155,648 for bf16; one vector more takes the other kernel again)
        fb.fopd_set_option("k14_regs", 1 if threads == 0 else 0)
        fb.fopd_set_option("k14_threads", threads if threads else 256)
        fb.fopd_set_option("k14_rows_per_cu", rows_per_cu)
        one = _pass_for(w)
        one.dlogits.fill_(5.0)
        call(one, 0, T, None, None, one.logp, one.dlogits, None)            # counts taken from the mask
        _sync_ok(one)
        in_regs = threads == 0 and 2048 < V // (8 if dtype == "bf16" else 4) <= 19456
        def same(x, y_):
            if threads == 256 or (threads == 0 and not in_regs):
                return torch.equal(x, y_)
            xd, yd = np64(x), np64(y_)
            if dtype == "bf16":
                return bool(np.all(np.abs(xd - yd) <= orc.bf16_ulp(yd))) and float(np.mean(xd == yd)) > 0.9
            # fp32 storage shows the last place of lse in every entry of a row
            return bool(np.all(np.abs(xd - yd) <= 1e-5 * np.abs(yd) + 1e-30))

        if in_regs:
            # another summation order moves lp in its last place, and with it the coefficient of a row whose
            # A_t - lambda rho_t delta_t nearly cancels by more than a relative bound allows: compare with the oracle
            oref, z64, y64 = _scored_reference(w, hp, np64(f_gpu), np64(n_gpu), 0.5)
            eps_c = coef_uncertainty(oref, hp, 0.5, B, np64(w["mask"]))
            check_grad_rows(np64(one.dlogits)[:, :V], z64, y64, oref["lse"], oref["coef"], eps_c, dtype)
        else:
            assert same(one.dlogits[:, :V], ref.dlogits[:, :V])
        if ld > V:
            assert bool((one.dlogits[:, V:] == 5.0).all())
        assert torch.equal(one.weights, ref.weights)
        assert torch.equal(one.logp, st.logp) or ((threads not in (256,) or in_regs) and
                                                  torch.allclose(one.logp, st.logp, rtol=2e-6, atol=2e-6))
        assert abs(float(one.loss) - float(ref.loss)) <= 2e-6 * abs(float(ref.loss)) + 1e-12
        # a row range that starts inside a sample, output aliased onto the input, no log-prob output
        a, b = 3, T - 2
        z = w["logits"].clone()
        two = _pass_for(w, alloc_dlogits=False)
        fb.fopd_loss_fwd_bwd(z[a:b], two.dt, b - a, V, ld, w["token_ids"][a:b], w["mask"][a:b],
                             w["behav_logp"][a:b], w["teacher_logp"][a:b], None, w["seq_lens"], w["lag"], B, hp,
                             f_gpu, n_gpu, None, a, None, None, 0.5, two.loss, None, None, None, z[a:b], two.workspace)
        _sync_ok(two)
        if in_regs:
            assert torch.equal(z[a:b, :V], one.dlogits[a:b, :V])           # the same kernel on a row range, in place
        else:
            assert same(z[a:b, :V], ref.dlogits[a:b, :V])
        assert torch.equal(z[:a], w["logits"][:a]) and torch.equal(z[b:], w["logits"][b:])
    finally:
        fb.fopd_set_option("k14_threads", 256)
        fb.fopd_set_option("k14_rows_per_cu", 6)
        fb.fopd_set_option("k14_regs", 1)


@pytest.mark.parametrize("dtype,V,ld,workload", [("bf16", 16392, 16392, "tooluse"), ("bf16", 151936, 151936, "tooluse"),
                                                 ("bf16", 5003, 5008, "tooluse"), ("f32", 9001, 9004, "tooluse"),
                                                 ("bf16", 20000, 20000, "two_sets")])
def test_single_read_call_returns_rows_at_unit_weight(dtype, V, ld, workload):
    """fopd_loss_fwd_bwd_unit reads each row once and returns u_t with dL/dz_t = w_i u_t.  Against the oracle:
    the rows at unit weight (2 ulp of the storage type plus the coefficient floor of the log-prob error alone:
    no score enters u_t), log-probs, scores, weights and loss; a gated sample keeps non-zero rows under weight 0,
    an invalid one has zero rows; and weight x row reproduces the two-read call's gradient."""
    _say("single-read call, rows at unit weight: %s V=%d (%s)" % (dtype, V, workload))
    if workload == "two_sets":
        w = wl.generate("tooluse", DEV, seed=41, B=6, turns=2, obs_lo=2, obs_hi=5, resp_lo=3, resp_hi=8, V=V, ld=ld,
                        dtype=dtype, boost=4, lag_lo=0, lag_hi=30, row_block=32, aligned_split=(0.3, 0.3))
    else:
        w = wl.generate("tooluse", DEV, seed=17, B=6, turns=2, obs_lo=2, obs_hi=5, resp_lo=3, resp_hi=9, V=V, ld=ld,
                        dtype=dtype, boost=min(4, V), lag_lo=0, lag_hi=30, row_block=32)
    T, B = w["T"], w["B"]
    hp, gs = (1.0, 1.0, 0.05, 0.3), 0.75
    ref = oracle_full(w, hp, gs, want_dlogits=True, unit_rows=True)
    lp = _pass_for(w)
    lp.dlogits.fill_(7.0)
    fb.fopd_loss_fwd_bwd_unit(w["logits"], lp.dt, T, V, ld, w["token_ids"], w["mask"], w["behav_logp"],
                              w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp, gs, lp.loss,
                              lp.freshness, lp.weights, lp.logp, lp.dlogits, lp.workspace)
    _sync_ok(lp)
    live = np64(w["mask"]) != 0
    assert_close("logp", np64(lp.logp), ref["logp"], atol=1e-4)
    assert_close("logp (relative)", np64(lp.logp)[live], ref["logp"][live], rtol=1e-5, atol=2e-6)
    assert_close("freshness", np64(lp.freshness), ref["freshness"], rtol=1e-5)
    assert_close("weights", np64(lp.weights), ref["weights"], atol=1e-5 * ref["freshness"] + 1e-12)
    assert abs(float(lp.loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-12, (float(lp.loss), ref["loss"])
    valid = np.minimum(ref["n_train"], ref["n_roll"]) > 0
    unit_ref = dict(ref, weights=valid.astype(np.float64), freshness=np.zeros(B))
    eps_c = coef_uncertainty(unit_ref, hp, gs, B, np64(w["mask"]))
    got = np64(lp.dlogits)
    y = ref["gather_idx"] - np.arange(T) * ld
    check_grad_rows(got[:, :V], np64(w["logits"])[:, :V], y, ref["lse"], ref["coef_unit"], eps_c, dtype)
    if ld > V:
        assert bool((lp.dlogits[:, V:] == 7.0).all())
    cu = ref["cu_seqlens"]
    gated = [i for i in range(B) if valid[i] and ref["weights"][i] == 0.0]
    assert gated and bool(np.any(ref["weights"] > 0))
    for i in gated:
        assert float(lp.weights[i]) == 0.0 and bool(np.any(got[cu[i]:cu[i + 1], :V] != 0.0))
    for i in range(B):
        if not valid[i]:
            assert bool(np.all(got[cu[i]:cu[i + 1], :V] == 0.0))
    # weight x row against the two-read call: the product is rounded a second time
    two = _pass_for(w)
    two.loss_fwd_bwd(w, hp, gs)
    _sync_ok(two)
    w_rows = np.repeat(np64(lp.weights), np64(w["seq_lens"]).astype(np.int64))[:, None]
    full = np64(two.dlogits)[:, :V]
    ulp = orc.bf16_ulp(full) if dtype == "bf16" else np.abs(full) * 2.0 ** -23
    prod = w_rows * got[:, :V]
    eps_rows = coef_uncertainty(ref, hp, gs, B, np64(w["mask"]))[:, None] * 2.0
    assert bool(np.all(np.abs(prod - full) <= 2.0 * ulp + eps_rows + 1e-30))
    assert abs(float(two.loss) - float(lp.loss)) <= 2e-6 * abs(float(two.loss)) + 1e-12
    assert torch.allclose(two.weights, lp.weights, rtol=2e-6, atol=1e-7)


def test_single_read_call_random_shapes_sweep():
    """Twenty seeded random problems through fopd_loss_fwd_bwd_unit: rows short enough for the kernel that re-reads
    a row and long enough for the one that holds it in registers, both storage types, one or two aligned sets, lags
    (some gated), hyper-parameters and upstream scale."""
    rs = np.random.RandomState(88)
    for case in range(20):
        dtype = "bf16" if rs.rand() < 0.7 else "f32"
        per = 8 if dtype == "bf16" else 4
        V = int(rs.choice([2, 9, 64, 1000, 4096, 10007, 16392, 20000, 40000, 77777]))
        ld = ((V + per - 1) // per) * per + per * int(rs.randint(0, 3))
        B = int(rs.randint(1, 6))
        hp = (float(rs.choice([0.0, 0.5, 1.0, 2.0])), float(rs.choice([0.0, 1.0])),
              float(rs.choice([0.0, 0.05, 0.2])), float(rs.choice([0.0, 0.1, 1.0])))
        gs = float(rs.choice([1.0, 0.125, -2.0]))
        split = dict(aligned_split=(0.3, 0.3)) if case % 3 == 2 else {}
        _say("single-read random case %d: %s V=%d ld=%d B=%d hp=%s g=%g" % (case, dtype, V, ld, B, hp, gs))
        w = wl.generate("tooluse", DEV, seed=4000 + case, B=B, turns=int(rs.randint(1, 4)), obs_lo=0,
                        obs_hi=int(rs.randint(0, 5)), resp_lo=0, resp_hi=int(rs.randint(1, 9)), V=V, ld=ld, dtype=dtype,
                        boost=min(3, V), lag_lo=0, lag_hi=int(rs.choice([0, 3, 25])),
                        stale_sigma=float(rs.choice([0.0, 0.1])), row_block=64, **split)
        T = w["T"]
        if T == 0:
            continue
        ref = oracle_full(w, hp, gs, want_dlogits=True, unit_rows=True)
        lp = _pass_for(w)
        lp.dlogits.fill_(7.0)
        fb.fopd_loss_fwd_bwd_unit(w["logits"], lp.dt, T, V, ld, w["token_ids"], w["mask"], w["behav_logp"],
                                  w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp, gs, lp.loss,
                                  lp.freshness, lp.weights, lp.logp, lp.dlogits, lp.workspace)
        _sync_ok(lp)
        live = np64(w["mask"]) != 0
        assert_close("logp", np64(lp.logp)[live], ref["logp"][live], rtol=1e-5, atol=2e-6)
        assert_close("freshness", np64(lp.freshness), ref["freshness"], rtol=1e-5)
        assert_close("weights", np64(lp.weights), ref["weights"], atol=1e-5 * ref["freshness"] + 1e-12)
        # L = mean_i w_i (l_i + lambda D_i): w_i = f_i - xi carries the absolute 1e-5 f_i of its score (case 9 here:
        # f = 0.0504 against xi = 0.05, so w is known to 1e-3 of itself), and l_i is a mean of differences of fp32
        # log-probs, good to 1e-6 absolute
        per_sample = (1e-5 * ref["freshness"] * np.abs(ref["ell"] + hp[3] * ref["D_roll"]) * (ref["weights"] > 0)
                      + 1e-6 * ref["weights"])
        loss_tol = 1e-5 * abs(ref["loss"]) + float(np.mean(per_sample)) + 1e-12
        assert abs(float(lp.loss) - ref["loss"]) <= loss_tol, (float(lp.loss), ref["loss"])
        valid = np.minimum(ref["n_train"], ref["n_roll"]) > 0
        unit_ref = dict(ref, weights=valid.astype(np.float64), freshness=np.zeros(B))
        eps_c = coef_uncertainty(unit_ref, hp, gs, B, np64(w["mask"]))
        y = ref["gather_idx"] - np.arange(T) * ld
        check_grad_rows(np64(lp.dlogits)[:, :V], np64(w["logits"])[:, :V], y, ref["lse"], ref["coef_unit"], eps_c, dtype)
        if ld > V:
            assert bool((lp.dlogits[:, V:] == 7.0).all())


def test_single_read_call_without_a_mask_counts_every_row():
    """A NULL mask means that every row is in both aligned sets, and a NULL stale teacher log-prob means
    D^sup = 0: checked against the oracle given a mask of ones and the fresh teacher log-probs as the stale ones."""
    _say("single-read call, no mask and no stale teacher log-probs")
    w = wl.generate("tooluse", DEV, seed=23, B=5, turns=2, obs_lo=0, obs_hi=0, resp_lo=3, resp_hi=9, V=16392,
                    ld=16392, dtype="bf16", boost=4, lag_lo=0, lag_hi=30, row_block=32)
    T, B, V, ld = w["T"], w["B"], w["V"], w["ld"]
    hp, gs = (1.0, 1.0, 0.05, 0.3), 1.0
    full = dict(w, mask=torch.ones(T, dtype=torch.uint8, device=DEV), teacher_logp_stale=w["teacher_logp"])
    ref = oracle_full(full, hp, gs, want_dlogits=True, unit_rows=True)
    assert float(np.max(np.abs(ref["D_sup"]))) == 0.0
    lp = _pass_for(w)
    fb.fopd_loss_fwd_bwd_unit(w["logits"], lp.dt, T, V, ld, w["token_ids"], None, w["behav_logp"], w["teacher_logp"],
                              None, w["seq_lens"], w["lag"], B, hp, gs, lp.loss, lp.freshness, lp.weights, lp.logp,
                              lp.dlogits, lp.workspace)
    _sync_ok(lp)
    assert_close("logp", np64(lp.logp), ref["logp"], rtol=1e-5, atol=2e-6)
    assert_close("freshness", np64(lp.freshness), ref["freshness"], rtol=1e-5)
    assert_close("weights", np64(lp.weights), ref["weights"], atol=1e-5 * ref["freshness"] + 1e-12)
    assert abs(float(lp.loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-12, (float(lp.loss), ref["loss"])
    valid = np.minimum(ref["n_train"], ref["n_roll"]) > 0
    unit_ref = dict(ref, weights=valid.astype(np.float64), freshness=np.zeros(B))
    eps_c = coef_uncertainty(unit_ref, hp, gs, B, np.ones(T))
    y = ref["gather_idx"] - np.arange(T) * ld
    check_grad_rows(np64(lp.dlogits)[:, :V], np64(w["logits"])[:, :V], y, ref["lse"], ref["coef_unit"], eps_c, "bf16")


# ---------------------------------------------------------------------------------------
# full-vocabulary rollout drift (the diagnostic as printed in the paper)
# ---------------------------------------------------------------------------------------

FULL_KL_CASES = {
    "reasoning": dict(B=6, len_lo=12, len_hi=30, V=151936, stale_logit_sigma=0.03),
    "tooluse": dict(B=4, turns=2, obs_lo=2, obs_hi=6, resp_lo=4, resp_hi=10, V=5003, ld=5008, stale_logit_sigma=0.05,
                    lag_hi=24),
    "coding": dict(B=2, total_len=48, resp_lo=6, resp_hi=14, obs_lo=3, obs_hi=8, V=40000, stale_logit_sigma=0.02),
    "tiny": dict(B=4, len_lo=9, len_hi=9, V=4097, ld=4100, stale_logit_sigma=0.04),
}


@pytest.mark.parametrize("name", sorted(FULL_KL_CASES))
def test_full_vocabulary_drift_variant(name):
    _say("full-vocabulary KL variant on a %s replica" % name)
    w = wl.generate(name, DEV, seed=21, row_block=32, **FULL_KL_CASES[name])
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]
    hp, g = (1.0, 1.0, 0.05, 0.5), 2.0
    z, zs = np64(w["logits"])[:, :V], np64(w["logits_stale"])[:, :V]
    ref = orc.fopd_loss_fwd_bwd_full_kl(z, zs, np64(w["token_ids"]), np64(w["mask"]), np64(w["teacher_logp"]),
                                        np64(w["teacher_logp_stale"]), np64(w["seq_lens"]), np64(w["lag"]),
                                        hp[0], hp[1], hp[2], hp[3], g, out_dtype=w["dtype"])
    lp = _pass_for(w)
    kl = torch.empty(T, device=DEV)
    dlse = torch.empty(T, device=DEV)
    lp.dlogits.fill_(4.0)
    fb.fopd_loss_fwd_bwd_full_kl(w["logits"], w["logits_stale"], lp.dt, T, V, ld, ld, w["token_ids"], w["mask"],
                                 w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp,
                                 None, None, None, 0, None, None, None, None, g,
                                 lp.loss, lp.freshness, lp.weights, lp.logp, kl, lp.dlogits, lp.workspace)
    _sync_ok(lp)
    live = np64(w["mask"]) != 0
    assert_close("logp", np64(lp.logp), ref["logp"], atol=1e-4)
    # fp32 sums over the vocabulary: 2e-5 relative plus 3e-8 absolute on the per-row KL
    assert_close("roll_kl", np64(kl), ref["roll_kl"], rtol=2e-5, atol=KL_ROW_ATOL)
    assert not np.any(np64(kl)[~live]) and np.all(np64(kl) >= 0)
    assert_close("freshness", np64(lp.freshness), ref["freshness"], rtol=1e-5)
    assert_close("weights", np64(lp.weights), ref["weights"], atol=1e-5 * ref["freshness"] + 1e-12)
    assert abs(float(lp.loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-12
    sample_of = np.repeat(np.arange(B), np64(w["seq_lens"]))
    check_grad_rows_full_kl(np64(lp.dlogits)[:, :V], z, zs, np64(w["token_ids"]), ref, range(T), hp, g, B, sample_of,
                            w["dtype"])
    if ld > V:
        assert bool((lp.dlogits[:, V:] == 4.0).all())
    # staged: drift pass on its own, then the scores with roll_kl in place of the sampled estimator
    st = _pass_for(w, alloc_dlogits=False)
    fb.fopd_rollout_kl(w["logits"], w["logits_stale"], st.dt, T, V, ld, ld, w["token_ids"], w["mask"], kl, st.logp,
                       st.lse, dlse, None, st.workspace)
    fb.fopd_freshness_score(st.logp, None, kl, None, w["teacher_logp"], w["teacher_logp_stale"], w["mask"], w["seq_lens"],
                            w["lag"], T, B, hp, st.cu_seqlens, st.n_train, st.n_roll, st.D_roll, st.D_sup, st.ell, st.cover,
                            st.cover_roll, st.freshness, st.agg, st.workspace)
    _sync_ok(st)
    assert torch.equal(st.logp, lp.logp) and torch.equal(st.freshness, lp.freshness)
    assert_close("D_roll", np64(st.D_roll), ref["D_roll"], rtol=2e-5, atol=3e-8)
    assert_close("lse", np64(st.lse), ref["lse"], atol=1e-4)
    assert_close("dlse", np64(dlse), (ref["lse"] - ref["lse_stale"]) * live, atol=2e-6, rtol=1e-5)
    # a lag-0 sample has identical stale logits: exactly zero drift, fresh score
    for i in np.flatnonzero((np64(w["lag"]) == 0) & (ref["n_train"] > 0)):
        assert float(st.D_roll[i]) == 0.0
    # in place over the current logits
    zc = w["logits"].clone()
    fb.fopd_loss_fwd_bwd_full_kl(zc, w["logits_stale"], lp.dt, T, V, ld, ld, w["token_ids"], w["mask"],
                                 w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp,
                                 None, None, None, 0, None, None, None, None, g,
                                 lp.loss, None, None, None, None, zc, lp.workspace)
    _sync_ok(lp)
    assert torch.equal(zc[:, :V], lp.dlogits[:, :V])


def test_replay_from_a_hip_graph():
    """The calls enqueue kernels and device copies only, so a caller may capture them in a HIP graph (worth
    it for small problems, where the six launches of a step cost more than the kernels).  Replays,
    with eager work and synchronisations in between, must reproduce the eager bits."""
    _say("HIP graph capture and replay of the fused step and of the scores-supplied step")
    w = wl.generate("tiny", DEV, seed=4)
    eager = _pass_for(w)
    eager.loss_fwd_bwd(w, HP)
    torch.cuda.synchronize()
    f_in = eager.freshness.clone()
    sc = _pass_for(w)
    fb.fopd_loss_fwd_bwd(w["logits"], sc.dt, w["T"], w["V"], w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                         w["teacher_logp"], None, w["seq_lens"], w["lag"], w["B"], HP, f_in, None, None, 0, None,
                         None, 1.0, sc.loss, None, sc.weights, sc.logp, sc.dlogits, sc.workspace)   # also warms the kernel up
    torch.cuda.synchronize()
    g1, g2 = _pass_for(w), _pass_for(w)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        g1.loss_fwd_bwd(w, HP)
        fb.fopd_loss_fwd_bwd(w["logits"], g2.dt, w["T"], w["V"], w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                             w["teacher_logp"], None, w["seq_lens"], w["lag"], w["B"], HP, f_in, None, None, 0, None,
                             None, 1.0, g2.loss, None, g2.weights, g2.logp, g2.dlogits, g2.workspace)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        g1.dlogits.fill_(float(rep))                 # eager work between the replays
        g2.dlogits.fill_(float(rep))
        g1.loss.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g1.dlogits, eager.dlogits) and torch.equal(g1.loss, eager.loss)
        assert torch.equal(g1.freshness, eager.freshness) and torch.equal(g1.logp, eager.logp)
        assert torch.equal(g2.dlogits, sc.dlogits) and torch.equal(g2.loss, sc.loss)
    _sync_ok(g1)
    _sync_ok(g2)


@pytest.mark.parametrize("dtype,V,seed", [("bf16", 20011, 3), ("f32", 9006, 4), ("bf16", 155648, 5), ("bf16", 16392, 6),
                                          ("bf16", 155659, 7), ("f32", 160003, 8), ("bf16", 262144, 9)])
def test_gradient_kernel_in_the_row_in_registers_shape_gives_the_same_bits(dtype, V, seed):
    """The fused step (log-sum-exp pass, scores, gradient pass) with the gradient kernel in its two launch shapes:
    one 256-lane workgroup per row, and 1024-lane workgroups that walk rows holding each in registers between its
    loads and its stores (masked, gated, live and invalid rows in any order; more rows than workgroups; a ragged row
    end; rows longer than the registers hold, which go in two or three runs; the gradient written over the logits)."""
    _say("gradient kernel, row-in-registers shape against one workgroup per row: %s V=%d" % (dtype, V))
    w = wl.generate("tooluse", DEV, seed=seed, B=40, turns=3, obs_lo=0, obs_hi=9, resp_lo=1, resp_hi=24, V=V,
                    ld=(V + 7) // 8 * 8 + 8, dtype=dtype, boost=4, lag_lo=0, lag_hi=40, row_block=64,
                    aligned_split=(0.2, 0.2))
    assert w["T"] > 600
    hp = (1.0, 1.0, 0.05, 0.3)
    out = {}
    try:
        for shape in (0, 1):
            fb.fopd_set_option("k4_regs", shape)
            lp = _pass_for(w)
            lp.dlogits.fill_(3.0)
            lp.loss_fwd_bwd(w, hp)
            _sync_ok(lp)
            out[shape] = lp
    finally:
        fb.fopd_set_option("k4_regs", 1)
    assert torch.equal(out[0].dlogits, out[1].dlogits) and torch.equal(out[0].loss, out[1].loss)
    assert bool((out[1].dlogits[:, V:] == 3.0).all())                 # the row padding is not touched
    live = (out[1].weights > 0)
    assert bool(live.any()) and bool((~live).any()) and bool(out[1].dlogits[:, :V].any())
    # in place
    inplace = _pass_for(w, alloc_dlogits=False)
    logits = w["logits"].clone()
    fb.fopd_loss_fwd_bwd(logits, inplace.dt, w["T"], V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                         w["teacher_logp"], None, w["seq_lens"], w["lag"], w["B"], hp, None, None, None, 0, None, None,
                         1.0, inplace.loss, inplace.freshness, inplace.weights, inplace.logp, logits, inplace.workspace)
    _sync_ok(inplace)
    assert torch.equal(logits[:, :V], out[1].dlogits[:, :V])


@pytest.mark.parametrize("dtype,V,seed", [("bf16", 20008, 3), ("f32", 9004, 4), ("bf16", 155648, 5)])
def test_row_in_registers_kernel_walks_many_rows_per_workgroup(dtype, V, seed):
    """More rows than compute units, so that every workgroup of the row-in-registers kernel walks several rows
    (masked, gated, live and invalid ones in any order) and requests the next row while storing the current one.
    Compared with the kernel that re-reads the row (256 lanes, the bits of the separate kernels): another summation
    order, so entries may differ by one unit of the storage type; masked and gated rows are zero in both."""
    _say("row-in-registers kernel over many rows per workgroup: %s V=%d" % (dtype, V))
    w = wl.generate("tooluse", DEV, seed=seed, B=40, turns=3, obs_lo=0, obs_hi=9, resp_lo=1, resp_hi=24, V=V, ld=V,
                    dtype=dtype, boost=4, lag_lo=0, lag_hi=40, row_block=64, aligned_split=(0.2, 0.2))
    T, B = w["T"], w["B"]
    assert T > 600
    hp = (1.0, 1.0, 0.05, 0.3)
    st = _pass_for(w)
    st.token_logprobs(w)
    st.freshness_score(w, hp)
    _sync_ok(st)
    f_gpu, n_gpu, nr_gpu = st.freshness.clone(), st.n_train.clone(), st.n_roll.clone()
    assert bool((f_gpu < 0.05).any()) and bool((f_gpu > 0.05).any())

    def call(lp):
        lp.dlogits.fill_(3.0)
        fb.fopd_loss_fwd_bwd(w["logits"], lp.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                             w["teacher_logp"], None, w["seq_lens"], w["lag"], B, hp, f_gpu, n_gpu, nr_gpu, 0, None, None,
                             0.5, lp.loss, None, lp.weights, lp.logp, lp.dlogits, lp.workspace)
        _sync_ok(lp)

    regs, plain = _pass_for(w), _pass_for(w)
    call(regs)
    try:
        fb.fopd_set_option("k14_regs", 0)
        call(plain)
    finally:
        fb.fopd_set_option("k14_regs", 1)
    assert torch.equal(regs.weights, plain.weights)
    assert torch.allclose(regs.logp, plain.logp, rtol=2e-6, atol=2e-6)
    assert abs(float(regs.loss) - float(plain.loss)) <= 2e-6 * abs(float(plain.loss)) + 1e-12
    x, y_ = np64(regs.dlogits), np64(plain.dlogits)
    if dtype == "bf16":
        # a coefficient that nearly cancels moves by more than one unit when lp moves in its last place: rows
        # are compared relative to their own largest entry as well
        # (a fresh sample's roll-only row has delta = lp - lb = 0 up to that last place: its whole row is ~1e-7 of
        # the others, or exactly zero, hence the bound relative to the largest entry of the matrix)
        row_scale = np.max(np.abs(y_), axis=1, keepdims=True)
        ok = ((np.abs(x - y_) <= orc.bf16_ulp(y_)) | (np.abs(x - y_) <= 2e-2 * row_scale)
              | (np.abs(x - y_) <= 1e-6 * np.max(np.abs(y_))))
        assert bool(np.all(ok)) and float(np.mean(x == y_)) > 0.97
    else:
        # fp32 storage shows the last place of lse in every entry, and a nearly cancelling coefficient moves more
        row_scale = np.max(np.abs(y_), axis=1, keepdims=True)
        ok = ((np.abs(x - y_) <= 1e-5 * np.abs(y_)) | (np.abs(x - y_) <= 2e-2 * row_scale)
              | (np.abs(x - y_) <= 1e-6 * np.max(np.abs(y_))))
        assert bool(np.all(ok))
        close = np.abs(x - y_) <= 1e-5 * np.abs(y_) + 1e-30
        assert float(np.mean(close)) > 0.97
    # rows of masked tokens and of gated or invalid samples: exactly zero
    wrow = np.repeat(np64(regs.weights), np64(w["seq_lens"]).astype(np.int64))
    dead = (np64(w["mask"]) == 0) | (wrow == 0.0)
    assert dead.any() and not np.any(x[dead])
    # the number of workgroups that share the rows does not change a bit of the result
    try:
        for grid in (1, 7, 4096):
            fb.fopd_set_option("k14_regs_grid", grid)
            again = _pass_for(w)
            call(again)
            assert torch.equal(again.dlogits, regs.dlogits) and torch.equal(again.logp, regs.logp), grid
            assert torch.equal(again.loss, regs.loss) and torch.equal(again.weights, regs.weights), grid
    finally:
        fb.fopd_set_option("k14_regs_grid", 0)


def test_replay_of_the_row_in_registers_kernel_from_a_hip_graph():
    """The same for the kernel that holds a row in registers (rows of 2049 16-byte vectors), in both of its uses:
    the scores-supplied call and the single-read call."""
    _say("HIP graph capture and replay: scores-supplied and single-read calls, rows held in registers")
    w = wl.generate("tooluse", DEV, seed=23, B=5, turns=2, obs_lo=2, obs_hi=5, resp_lo=3, resp_hi=9, V=16392, ld=16392,
                    dtype="bf16", boost=4, lag_lo=0, lag_hi=30, row_block=32)
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]

    def unit(lp):
        fb.fopd_loss_fwd_bwd_unit(w["logits"], lp.dt, T, V, ld, w["token_ids"], w["mask"], w["behav_logp"],
                                  w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, HP, 1.0, lp.loss,
                                  lp.freshness, lp.weights, lp.logp, lp.dlogits, lp.workspace)

    def scored(lp, f_in):
        fb.fopd_loss_fwd_bwd(w["logits"], lp.dt, T, V, ld, w["token_ids"], w["mask"], w["behav_logp"], w["teacher_logp"],
                             w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, HP, f_in, None, None, 0, None, None,
                             1.0, lp.loss, None, lp.weights, lp.logp, lp.dlogits, lp.workspace)

    e1, e2 = _pass_for(w), _pass_for(w)
    unit(e1)                                           # eager; also the first call outside any capture
    torch.cuda.synchronize()
    f_in = e1.freshness.clone()
    scored(e2, f_in)
    torch.cuda.synchronize()
    g1, g2 = _pass_for(w), _pass_for(w)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        unit(g1)
        scored(g2, f_in)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        g1.dlogits.fill_(float(rep))
        g2.dlogits.fill_(float(rep))
        g1.loss.zero_()
        g1.weights.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g1.dlogits, e1.dlogits) and torch.equal(g1.loss, e1.loss) and torch.equal(g1.weights, e1.weights)
        assert torch.equal(g1.freshness, e1.freshness) and torch.equal(g1.logp, e1.logp)
        assert torch.equal(g2.dlogits, e2.dlogits) and torch.equal(g2.loss, e2.loss)
    _sync_ok(g1)
    _sync_ok(g2)


@pytest.mark.parametrize("name", ["reasoning", "coding", "tiny"])
def test_full_teacher_distribution_variant(name):
    """Token loss = KL(student || teacher) from the teacher's full logits (here: the generator's second
    logits tensor plays the teacher), rollout drift from the sampled-token estimator."""
    _say("distribution-level teacher loss on a %s replica" % name)
    over = dict(FULL_KL_CASES[name], stale_logit_sigma=0.3)
    if name == "tiny":
        over["lags"] = [1, 2, 3, 30]                     # the last sample is gated
    w = wl.generate(name, DEV, seed=31, row_block=32, **over)
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]
    hp, g = (1.0, 1.0, 0.05, 0.5), 1.5
    z, zq = np64(w["logits"])[:, :V], np64(w["logits_stale"])[:, :V]
    # the generator's stored per-token teacher log-prob is used here as the stale-context one
    ref = orc.fopd_loss_fwd_bwd_full_teacher(z, zq, np64(w["token_ids"]), np64(w["mask"]), np64(w["behav_logp"]),
                                             np64(w["teacher_logp"]), np64(w["seq_lens"]), np64(w["lag"]),
                                             hp[0], hp[1], hp[2], hp[3], g, out_dtype=w["dtype"])
    lp = _pass_for(w)
    kl = torch.empty(T, device=DEV)
    lp.dlogits.fill_(4.0)
    fb.fopd_loss_fwd_bwd_full_teacher(w["logits"], w["logits_stale"], lp.dt, T, V, ld, ld, w["token_ids"], w["mask"],
                                      w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp,
                                      None, None, None, 0, None, None, None, None, g, lp.loss,
                                      lp.freshness, lp.weights, lp.logp, kl, lp.dlogits, lp.workspace)
    _sync_ok(lp)
    assert_close("logp", np64(lp.logp), ref["logp"], atol=1e-4)
    assert_close("token_kl", np64(kl), ref["token_kl"], rtol=2e-5, atol=KL_ROW_ATOL)
    assert_close("freshness", np64(lp.freshness), ref["freshness"], rtol=1e-5)
    assert_close("weights", np64(lp.weights), ref["weights"], atol=1e-5 * ref["freshness"] + 1e-12)
    assert abs(float(lp.loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-12
    assert np.any(ref["D_sup"] > 0)                      # the teacher log-prob came out of the teacher logits
    sample_of = np.repeat(np.arange(B), np64(w["seq_lens"]))
    check_grad_rows_full_kl(np64(lp.dlogits)[:, :V], z, zq, np64(w["token_ids"]), ref, range(T), hp, g, B, sample_of,
                            w["dtype"], c2_scales_with_weight=True)
    if ld > V:
        assert bool((lp.dlogits[:, V:] == 4.0).all())


def test_profile_hooks_count_and_time_the_streaming_kernels():
    w = wl.generate("tiny", DEV, seed=5)
    lp = _pass_for(w)
    lp.loss_fwd_bwd(w, HP)
    torch.cuda.synchronize()
    fb.fopd_profile_reset()
    fb.fopd_profile_enable(True)
    try:
        for _ in range(3):
            lp.loss_fwd_bwd(w, HP)
        lp.token_logprobs(w)
    finally:
        fb.fopd_profile_enable(False)
    lp.loss_fwd_bwd(w, HP)                              # not recorded any more
    ms0, n0 = fb.fopd_profile_read(0)
    ms1, n1 = fb.fopd_profile_read(1)
    ms2, n2 = fb.fopd_profile_read(2)
    assert (n0, n1, n2) == (4, 3, 0) and ms0 > 0.0 and ms1 > 0.0 and ms2 == 0.0
    assert ms0 < 1000.0 and ms1 < 1000.0
    fb.fopd_profile_reset()
    assert fb.fopd_profile_read(0) == (0.0, 0)


def test_device_side_error_flags():
    _say("device flags: token range, segments, lag")
    w = wl.generate("reasoning", DEV, seed=12, B=3, len_lo=4, len_hi=6, V=512)
    good = _pass_for(w)
    good.loss_fwd_bwd(w, HP)
    _sync_ok(good)
    # token id out of range: flagged, row treated as masked, other rows unchanged
    bad = dict(w, token_ids=w["token_ids"].clone())
    bad["token_ids"][2] = 512
    bad["token_ids"][3] = -1
    lp = _pass_for(w)
    lp.token_logprobs(bad)
    st, flags = lp.status()
    assert st == 6 and flags == 1
    assert float(lp.logp[2]) == 0.0 and float(lp.logp[3]) == 0.0
    keep = [t for t in range(w["T"]) if t not in (2, 3)]
    assert torch.equal(lp.logp[keep], good.logp[keep])
    fb.fopd_workspace_init(lp.workspace)
    assert lp.status() == (0, 0)
    # lengths that do not add up to T
    bad = dict(w, seq_lens=w["seq_lens"].clone())
    bad["seq_lens"][0] += 1
    lp.loss_fwd_bwd(bad, HP)
    assert lp.status()[0] == 7
    fb.fopd_workspace_init(lp.workspace)
    bad = dict(w, lag=w["lag"].clone())
    bad["lag"][1] = -2
    lp.token_logprobs(w)
    lp.freshness_score(bad, HP)
    assert lp.status() == (8, 4)
    # ... and the sample with the negative lag is invalid: zero score, zero coverage, zero weight even with a
    # negative gate threshold, zero gradient rows; the other samples are untouched
    assert float(lp.freshness[1]) == 0.0 and float(lp.cover[1]) == 0.0 and float(lp.cover_roll[1]) == 0.0
    assert float(lp.freshness[0]) == float(good.freshness[0]) and float(lp.freshness[2]) == float(good.freshness[2])
    assert abs(float(lp.agg[0]) - (float(good.freshness[0]) + float(good.freshness[2])) / 3) < 1e-6
    fb.fopd_workspace_init(lp.workspace)
    lp.loss_fwd_bwd(bad, (1.0, 1.0, -0.5, 0.1))
    assert lp.status() == (8, 4)
    cu = np.concatenate([[0], np.cumsum(w["seq_lens_host"])])
    assert float(lp.weights[1]) == 0.0 and float(lp.weights[0]) > 0.5
    assert not bool(lp.dlogits[cu[1]:cu[2]].any()) and bool(lp.dlogits[cu[0]:cu[1]].any())
    assert bool(torch.isfinite(lp.dlogits.float()).all()) and bool(torch.isfinite(lp.loss).all())
    # a mask that names two different aligned sets, chunk call with one count array only: flagged, those rows dropped
    fb.fopd_workspace_init(lp.workspace)
    m2 = w["mask"].clone()
    m2[1] = 2
    m2[4] = 3
    st = _pass_for(w)
    st.token_logprobs(w)
    st.freshness_score(dict(w, mask=m2), HP)
    _sync_ok(st)
    T, V, B = w["T"], w["V"], w["B"]
    for lse_in, logp_in in ((st.lse, st.logp), (None, None)):       # gradient kernel alone / both passes in one kernel
        fb.fopd_workspace_init(lp.workspace)
        lp.dlogits.fill_(1.0)
        fb.fopd_loss_fwd_bwd(w["logits"], lp.dt, T, V, w["ld"], w["token_ids"], m2, w["behav_logp"], w["teacher_logp"],
                             None, w["seq_lens"], w["lag"], B, HP, st.freshness, st.n_train, None, 0, lse_in, logp_in,
                             1.0, lp.loss, None, lp.weights, None, lp.dlogits, lp.workspace)
        assert lp.status() == (10, 8)
        assert fb.fopd_flags_status(8) == 10 and fb.fopd_flags_status(0) == 0 and fb.fopd_flags_status(9) == 6
        assert not bool(lp.dlogits[1].any()) and not bool(lp.dlogits[4].any()) and bool(lp.dlogits[0].any())
    # with both count arrays the same call is clean
    fb.fopd_workspace_init(lp.workspace)
    fb.fopd_loss_fwd_bwd(w["logits"], lp.dt, T, V, w["ld"], w["token_ids"], m2, w["behav_logp"], w["teacher_logp"],
                         None, w["seq_lens"], w["lag"], B, HP, st.freshness, st.n_train, st.n_roll, 0, st.lse, st.logp,
                         1.0, lp.loss, None, lp.weights, None, lp.dlogits, lp.workspace)
    _sync_ok(lp)
    assert bool(lp.dlogits[1].any()) and bool(lp.dlogits[4].any())


def test_upstream_scale_and_lambda():
    w = wl.generate("tiny", DEV, seed=2, B=3, len_lo=7, len_hi=7, V=640)
    _compare_everything(w, (0.7, 0.0, 0.1, 0.0), grad_scale=0.25, staged=False)
    _compare_everything(w, (0.0, 2.0, 0.0, 2.0), grad_scale=-1.0, staged=False)


def test_ablation_arms_are_parameter_settings():
    """The ablation arms of App. B as plain settings of the same calls: lag-only scoring
    (alpha = beta = 0), weighting without the anchor (lambda = 0), and the anchor without weighting
    (scores supplied as 1 with xi = 0, so that every valid sample has weight 1)."""
    _say("ablation arms")
    w = wl.generate("coding", DEV, seed=21, B=4, total_len=48, resp_lo=5, resp_hi=12, obs_lo=2, obs_hi=7, V=9001, ld=9008)
    _compare_everything(w, (0.0, 0.0, 0.05, 0.1), grad_scale=1.0, staged=False)       # lag-only
    _compare_everything(w, (1.0, 1.0, 0.05, 0.0), grad_scale=1.0, staged=True)        # weighting-only
    T, V, B = w["T"], w["V"], w["B"]
    hp = (1.0, 1.0, 0.0, 0.4)
    ones = torch.ones(B, dtype=torch.float32, device=DEV)
    sc = _pass_for(w)
    fb.fopd_loss_fwd_bwd(w["logits"], sc.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                         w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp,
                         ones, None, None, 0, None, None, 1.0, sc.loss, sc.freshness, sc.weights, sc.logp,
                         sc.dlogits, sc.workspace)
    _sync_ok(sc)
    n_used = orc.trainable_counts(np64(w["mask"]), orc.segment_offsets(np64(w["seq_lens"])))
    ref, z, y = _scored_reference(w, hp, np.ones(B), n_used, 1.0)
    assert np.array_equal(np64(sc.weights), (n_used > 0).astype(np.float64))
    eps_c = coef_uncertainty(ref, hp, 1.0, B, np64(w["mask"]))
    check_grad_rows(np64(sc.dlogits)[:, :V], z, y, ref["lse"], ref["coef"], eps_c, w["dtype"])
    L = float(np.sum(ref["loss_terms"]))
    assert abs(float(sc.loss) - L) <= 1e-5 * abs(L)


# ---------------------------------------------------------------------------------------
# the benchmark's workload at full size, in the benchmark's launch configuration
# ---------------------------------------------------------------------------------------

def _oracle_sample(w, i, cu, hp, B, logits=None, block=2048):
    """Oracle values of one whole sample of a full-size workload, rows pulled to the host in blocks.
    `logits` replaces w["logits"] (a saved copy) when the call under test ran in place."""
    V = w["V"]
    a, b = int(cu[i]), int(cu[i + 1])
    src = w["logits"] if logits is None else logits
    off = 0 if logits is None else a
    mask = w["mask_host"][a:b]
    y = np64(w["token_ids"][a:b])
    lse, lpo = np.zeros(b - a), np.zeros(b - a)
    for s0 in range(a, b, block):
        e0 = min(s0 + block, b)
        l, p = orc.token_logprobs(np64(src[s0 - off:e0 - off, :V]), y[s0 - a:e0 - a], mask[s0 - a:e0 - a])
        lse[s0 - a:e0 - a], lpo[s0 - a:e0 - a] = l, p
    lb, lq = np64(w["behav_logp"][a:b]), np64(w["teacher_logp"][a:b])
    lqs = None if w["teacher_logp_stale"] is None else np64(w["teacher_logp_stale"][a:b])
    delta, rho, adv, k_roll, k_sup = orc.token_terms(lpo, lb, lq, lqs)
    cu1 = np.array([0, b - a], dtype=np.int64)
    D_roll, D_sup, ell, cover, n = orc.sample_statistics(lpo, lq, k_roll, k_sup, mask, cu1)
    f = orc.freshness_score(D_roll, D_sup, w["lag_host"][i:i + 1], n, hp[0], hp[1])
    wt = orc.freshness_weights(f, hp[2], n)
    coef = orc.grad_coefficients(delta, rho, adv, mask, cu1, n, wt, hp[3], 1.0, n_samples=B)
    ref = dict(coef=coef, cu_seqlens=cu1, n_train=n, freshness=f, weights=wt, adv=adv, rho=rho, delta=delta)
    eps_c = coef_uncertainty(ref, hp, 1.0, B, mask)
    # the same at unit sample weight (what the single-read call writes): no score enters
    ones = (n > 0).astype(np.float64)
    coef_unit = orc.grad_coefficients(delta, rho, adv, mask, cu1, n, ones, hp[3], 1.0, n_samples=B)
    eps_unit = coef_uncertainty(dict(ref, weights=ones, freshness=np.zeros(1)), hp, 1.0, B, mask)
    return dict(a=a, b=b, y=y, mask=mask, lse=lse, logp=lpo, D_roll=D_roll, D_sup=D_sup, ell=ell, cover=cover,
                n=n, f=f, w=wt, coef=coef, eps_c=eps_c, coef_unit=coef_unit, eps_unit=eps_unit)


def _check_sample(o, i, logp, lse, freshness, weights, st):
    live = o["mask"] != 0
    assert_close("logp sample %d" % i, np64(logp[o["a"]:o["b"]]), o["logp"], atol=1e-4)
    # lse is stored in fp32: one fp32 spacing at its magnitude on top of the 1e-4
    assert_close("lse sample %d" % i, np64(lse[o["a"]:o["b"]]), o["lse"],
                 atol=1e-4 + np.spacing(np.abs(o["lse"]).astype(np.float32)).astype(np.float64))
    assert not np.any(np64(logp[o["a"]:o["b"]])[~live])
    f = o["f"][0]
    assert abs(float(freshness[i]) - f) <= 1e-5 * f, (i, float(freshness[i]), f)
    assert abs(float(weights[i]) - o["w"][0]) <= 1e-5 * f
    if st is not None:
        assert_close("D_roll %d" % i, np64(st.D_roll[i:i + 1]), o["D_roll"], rtol=2e-5, atol=1e-9)
        assert_close("D_sup %d" % i, np64(st.D_sup[i:i + 1]), o["D_sup"], rtol=2e-5, atol=1e-9)
        assert_close("ell %d" % i, np64(st.ell[i:i + 1]), o["ell"], rtol=2e-5, atol=1e-6)
        assert_close("cover %d" % i, np64(st.cover[i:i + 1]), o["cover"], rtol=1e-6)
        assert int(st.n_train[i]) == int(o["n"][0])


def _check_sample_grad_rows(o, i, w, get_rows, picks, logits=None, unit=False):
    """picks: row numbers inside the sample; get_rows(global_rows) returns the GPU gradient rows."""
    V = w["V"]
    src = w["logits"] if logits is None else logits
    off = 0 if logits is None else o["a"]
    idx = torch.from_numpy(np.asarray(picks) + o["a"] - off).to(DEV)
    z = np64(src[idx][:, :V])
    got = np64(get_rows(np.asarray(picks) + o["a"]))[:, :V]
    coef, eps = ("coef_unit", "eps_unit") if unit else ("coef", "eps_c")
    check_grad_rows(got, z, o["y"][picks], o["lse"][picks], o[coef][picks], o[eps][picks], w["dtype"],
                    rows_label="s%d:" % i)


def _integers_everywhere(w, st, chunk=None):
    """cu_seqlens, n_train and gather_idx of every sample and row, bit for bit.  gather_idx is an offset
    from the matrix pointer of the call that wrote it, so with chunked calls it restarts per chunk."""
    cu = orc.segment_offsets(w["seq_lens_host"])
    assert np.array_equal(np64(st.cu_seqlens), cu)
    assert np.array_equal(np64(st.n_train), orc.trainable_counts(w["mask_host"], cu))
    ids = np64(w["token_ids"])
    if chunk is None:
        want = orc.gather_index(ids, w["ld"])
    else:
        want = np.concatenate([orc.gather_index(ids[a:a + chunk], w["ld"]) for a in range(0, w["T"], chunk)])
    assert np.array_equal(np64(st.gather_idx), want)
    return cu


def _row_properties(w, cu, dlogits_row, weights, n_rows=48, seed=1, expect_nonzero=True):
    """Properties that hold at any size: rows of gated or masked tokens are exactly zero, the others
    sum to ~0 (softmax minus one-hot) and are non-zero at the sampled token."""
    g = torch.Generator().manual_seed(seed)
    w_host = np64(weights)
    for t in torch.randint(0, w["T"], (n_rows,), generator=g).tolist():
        row = dlogits_row(t).double()
        i = int(np.searchsorted(cu, t, side="right") - 1)
        if w_host[i] == 0.0 or w["mask_host"][t] == 0:
            assert not bool(row.any()), "row %d must be zero" % t
        else:
            assert abs(float(row.sum())) <= 2.0 ** -7 * float(row.abs().sum()) + 1e-30
            if expect_nonzero:         # not with heavy tails: c (p_y - 1) underflows when p_y -> 1
                assert float(row[int(w["token_ids"][t])]) != 0.0


def _pick_samples(seq, min_samples, min_rows, prefer=None):
    order = list(np.argsort(seq, kind="stable"))
    if prefer:
        order = list(prefer) + [i for i in order if i not in prefer]
    chosen, rows = [], 0
    for i in order:
        chosen.append(int(i))
        rows += int(seq[i])
        if len(chosen) >= min_samples and rows >= min_rows:
            break
    return chosen, rows


def test_reasoning_full_size_sampled_parity():
    _say("reasoning at full size (B=64, V=151936): generating ...")
    w = wl.generate("reasoning", DEV, seed=0)
    T, V, B = w["T"], w["V"], w["B"]
    _say("T=%d rows, logits %.1f GB; running the fused call" % (T, T * V * 2 / 1e9))
    lp = _pass_for(w)
    lp.loss_fwd_bwd(w, HP)
    _sync_ok(lp)
    st = _pass_for(w, alloc_dlogits=False)
    st.token_logprobs(w)
    st.freshness_score(w, HP)
    _sync_ok(st)
    cu = _integers_everywhere(w, st)
    assert torch.equal(st.logp, lp.logp) and torch.equal(st.freshness, lp.freshness)
    # whole samples for the oracle: shortest first until at least 4 samples and 8k rows
    chosen, rows = _pick_samples(w["seq_lens_host"], 4, 8192)
    _say("oracle on samples %s (%d rows)" % (chosen, rows))
    oracle_samples = {}
    for i in chosen:
        o = oracle_samples[i] = _oracle_sample(w, i, cu, HP, B)
        _check_sample(o, i, lp.logp, st.lse, lp.freshness, lp.weights, st)
        picks = np.unique(np.linspace(0, o["b"] - o["a"] - 1, 6).astype(int))
        _check_sample_grad_rows(o, i, w, lambda rows_: lp.dlogits[torch.from_numpy(rows_).to(DEV)], picks)
        _say("sample %d ok (f=%.6f, w=%.6f)" % (i, o["f"][0], o["w"][0]))
    # the loss is the weighted mean of the per-sample terms the library itself reports
    w_gpu = np64(lp.weights)
    Ls = float(np.sum(w_gpu * (np64(st.ell) + HP[3] * np64(st.D_roll))) / B)
    assert abs(float(lp.loss) - Ls) <= 2e-6 * abs(Ls)
    _row_properties(w, cu, lambda t: lp.dlogits[t], lp.weights)
    assert_close("agg f", float(st.agg[0]), float(np.mean(np64(lp.freshness))), rtol=1e-6)
    # the call the benchmark also times: scores supplied, both passes over a row in one kernel, at this size
    _say("scores-supplied call at full size")
    f_in, first_loss, first_logp = lp.freshness.clone(), float(lp.loss), lp.logp.clone()
    lp.dlogits.fill_(2.0)
    lp.logp.fill_(2.0)
    fb.fopd_loss_fwd_bwd(w["logits"], lp.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                         w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, HP, f_in,
                         None, None, 0, None, None, 1.0, lp.loss, None, lp.weights, lp.logp, lp.dlogits, lp.workspace)
    _sync_ok(lp)
    # the row is held in registers by 1024 lanes: another summation order than the 256-lane pass, last place only
    assert torch.allclose(lp.logp, first_logp, rtol=2e-6, atol=2e-6)
    assert abs(float(lp.loss) - first_loss) <= 2e-6 * abs(first_loss)
    for i in chosen:
        o = oracle_samples[i]
        assert abs(float(lp.weights[i]) - o["w"][0]) <= 1e-5 * o["f"][0]
        picks = np.unique(np.linspace(0, o["b"] - o["a"] - 1, 6).astype(int))
        _check_sample_grad_rows(o, i, w, lambda rows_: lp.dlogits[torch.from_numpy(rows_).to(DEV)], picks)
    _row_properties(w, cu, lambda t: lp.dlogits[t], lp.weights, n_rows=24)
    # the whole pass with the logits read once, at this size: rows at unit sample weight, scores, weights, loss
    _say("single-read call at full size")
    lp.dlogits.fill_(2.0)
    lp.logp.fill_(2.0)
    lp.weights.fill_(2.0)
    lp.freshness.fill_(2.0)
    fb.fopd_loss_fwd_bwd_unit(w["logits"], lp.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                              w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, HP, 1.0, lp.loss,
                              lp.freshness, lp.weights, lp.logp, lp.dlogits, lp.workspace)
    _sync_ok(lp)
    assert torch.allclose(lp.logp, first_logp, rtol=2e-6, atol=2e-6)
    assert abs(float(lp.loss) - first_loss) <= 2e-6 * abs(first_loss)
    assert torch.allclose(lp.freshness, f_in, rtol=2e-6, atol=0.0)
    for i in chosen:
        o = oracle_samples[i]
        assert abs(float(lp.freshness[i]) - o["f"][0]) <= 1e-5 * o["f"][0]
        assert abs(float(lp.weights[i]) - o["w"][0]) <= 1e-5 * o["f"][0]
        picks = np.unique(np.linspace(0, o["b"] - o["a"] - 1, 6).astype(int))
        _check_sample_grad_rows(o, i, w, lambda rows_: lp.dlogits[torch.from_numpy(rows_).to(DEV)], picks, unit=True)
    _row_properties(w, cu, lambda t: lp.dlogits[t], torch.ones_like(lp.weights), n_rows=24)


def test_tooluse_full_size_sampled_parity():
    _say("tooluse at full size (B=32 x 8 turns, V=151936, masked observation spans): generating ...")
    w = wl.generate("tooluse", DEV, seed=0)
    T, V, B = w["T"], w["V"], w["B"]
    _say("T=%d rows (%d trainable), logits %.1f GB; fused call, gradient in place" % (T, w["n_trainable"], T * V * 2 / 1e9))
    chosen, rows = _pick_samples(w["seq_lens_host"], 2, 8192)
    cu0 = orc.segment_offsets(w["seq_lens_host"])
    saved = {i: w["logits"][int(cu0[i]):int(cu0[i + 1])].clone() for i in chosen}
    st = _pass_for(w, alloc_dlogits=False)
    st.token_logprobs(w)
    st.freshness_score(w, HP)
    _sync_ok(st)
    cu = _integers_everywhere(w, st)
    lp = _pass_for(w, alloc_dlogits=False)
    lp.loss_fwd_bwd(w, HP, dlogits=w["logits"])                  # in place: 75 GB instead of 150 GB
    _sync_ok(lp)
    assert torch.equal(st.logp, lp.logp) and torch.equal(st.freshness, lp.freshness)
    _say("oracle on samples %s (%d rows)" % (chosen, rows))
    for i in chosen:
        o = _oracle_sample(w, i, cu, HP, B, logits=saved[i])
        _check_sample(o, i, lp.logp, st.lse, lp.freshness, lp.weights, st)
        live = np.flatnonzero(o["mask"])
        dead = np.flatnonzero(o["mask"] == 0)
        picks = np.concatenate([live[np.linspace(0, len(live) - 1, 4).astype(int)], dead[:2]])
        _check_sample_grad_rows(o, i, w, lambda rows_: w["logits"][torch.from_numpy(rows_).to(DEV)], picks,
                                logits=saved[i])
        _say("sample %d ok (f=%.6f, w=%.6f, n=%d of %d)" % (i, o["f"][0], o["w"][0], o["n"][0], o["b"] - o["a"]))
    w_gpu = np64(lp.weights)
    Ls = float(np.sum(w_gpu * (np64(st.ell) + HP[3] * np64(st.D_roll))) / B)
    assert abs(float(lp.loss) - Ls) <= 2e-6 * abs(Ls)
    _row_properties(w, cu, lambda t: w["logits"][t], lp.weights)
    assert_close("agg cover", float(st.agg[1]), float(np.mean(np64(st.cover))), rtol=1e-6)


def test_tooluse_full_size_single_read_in_place():
    """The single-read call at full size on rows with masked spans, written in place: rows at unit weight for sampled
    rows of whole samples, masked rows zero, scores and weights against the oracle."""
    _say("tooluse at full size, single-read call in place: generating ...")
    w = wl.generate("tooluse", DEV, seed=0)
    T, V, B = w["T"], w["V"], w["B"]
    chosen, rows = _pick_samples(w["seq_lens_host"], 2, 8192)
    cu = orc.segment_offsets(w["seq_lens_host"])
    saved = {i: w["logits"][int(cu[i]):int(cu[i + 1])].clone() for i in chosen}
    lp = _pass_for(w, alloc_dlogits=False)
    fb.fopd_loss_fwd_bwd_unit(w["logits"], lp.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                              w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, HP, 1.0, lp.loss,
                              lp.freshness, lp.weights, lp.logp, w["logits"], lp.workspace)
    _sync_ok(lp)
    _say("oracle on samples %s (%d rows)" % (chosen, rows))
    for i in chosen:
        o = _oracle_sample(w, i, cu, HP, B, logits=saved[i])
        assert_close("logp sample %d" % i, np64(lp.logp[o["a"]:o["b"]]), o["logp"], atol=1e-4)
        f = o["f"][0]
        assert abs(float(lp.freshness[i]) - f) <= 1e-5 * f and abs(float(lp.weights[i]) - o["w"][0]) <= 1e-5 * f
        live = np.flatnonzero(o["mask"])
        dead = np.flatnonzero(o["mask"] == 0)
        picks = np.concatenate([live[np.linspace(0, len(live) - 1, 4).astype(int)], dead[:2]])
        _check_sample_grad_rows(o, i, w, lambda rows_: w["logits"][torch.from_numpy(rows_).to(DEV)], picks,
                                logits=saved[i], unit=True)
    _row_properties(w, cu, lambda t: w["logits"][t], torch.ones_like(lp.weights))


def test_coding_full_size_chunked_flow():
    _say("coding at full size (B=8 x 32768, V=151936), processed in chunks of 16384 rows: generating ...")
    w = wl.generate("coding", DEV, seed=0)
    T, V, B = w["T"], w["V"], w["B"]
    chunk = w["cfg"]["chunk"]
    assert T == 262144 and chunk == 16384
    full = _pass_for(w, alloc_dlogits=False)
    for a in range(0, T, chunk):                                  # phase 1: log-probs per chunk
        full.token_logprobs(w, rows=(a, a + chunk))
    full.freshness_score(w, HP)                                   # phase 2: scores over the O(T) arrays
    _sync_ok(full)
    cu = _integers_everywhere(w, full, chunk=chunk)
    lagh = w["lag_host"]                                          # smallest non-zero lag: D_sup > 0, not gated
    i = int(np.argmin(np.where(lagh > 0, lagh, 1 << 30)))
    _say("oracle on sample %d (%d rows, lag %d)" % (i, w["seq_lens_host"][i], w["lag_host"][i]))
    o = _oracle_sample(w, i, cu, HP, B)
    wts = torch.empty(B, device=DEV)
    _check_sample(o, i, full.logp, full.lse, full.freshness,
                  torch.clamp(full.freshness - HP[2], min=0.0), full)
    assert o["D_sup"][0] > 0
    # three more whole samples (one fresh, the others in lag order): log-probs, drift, loss term, score, weight
    others = [int(j) for j in np.argsort(lagh, kind="stable") if int(j) != i][:3]
    for j in others:
        _say("oracle on sample %d (lag %d): log-probs and per-sample values" % (j, lagh[j]))
        oj = _oracle_sample(w, j, cu, HP, B)
        _check_sample(oj, j, full.logp, full.lse, full.freshness, torch.clamp(full.freshness - HP[2], min=0.0), full)
    live = np.flatnonzero(o["mask"])
    picks = np.concatenate([live[np.linspace(0, len(live) - 1, 6).astype(int)], np.flatnonzero(o["mask"] == 0)[:2]])
    picks_global = set((picks + o["a"]).tolist())
    grads = {}
    dl = torch.empty(chunk, w["ld"], dtype=torch.bfloat16, device=DEV)
    total = 0.0
    part = torch.zeros(1, device=DEV)
    for a in range(0, T, chunk):                                  # phase 3: gradient per chunk
        b = a + chunk
        fb.fopd_loss_fwd_bwd(w["logits"][a:b], full.dt, chunk, V, w["ld"], w["token_ids"][a:b], w["mask"][a:b],
                             w["behav_logp"][a:b], w["teacher_logp"][a:b], w["teacher_logp_stale"][a:b],
                             w["seq_lens"], w["lag"], B, HP, full.freshness, full.n_train, None, a, full.lse[a:b],
                             full.logp[a:b], 1.0, part, None, wts, None, dl, full.workspace)
        total += float(part)
        for t in picks_global:
            if a <= t < b:
                grads[t] = dl[t - a].clone()
        if a == 0:
            _row_properties(dict(w, T=chunk), cu, lambda t: dl[t], wts, n_rows=16)
    _sync_ok(full)
    _check_sample_grad_rows(o, i, w, lambda rows_: torch.stack([grads[int(t)] for t in rows_]), picks)
    w_gpu = np64(wts)
    assert np.any(w_gpu == 0.0) and np.any(w_gpu > 0.0)           # lags up to 16: some samples gated
    Ls = float(np.sum(w_gpu * (np64(full.ell) + HP[3] * np64(full.D_roll))) / B)
    assert abs(total - Ls) <= 1e-5 * abs(Ls), (total, Ls)        # chunk losses add up to L


def test_largevocab_full_size_in_place():
    _say("largevocab at full size (B=16 x 16384, V=262144, heavy-tailed logits): generating ...")
    w = wl.generate("largevocab", DEV, seed=0)
    T, V, B = w["T"], w["V"], w["B"]
    _say("logits %.1f GB; gradient written in place" % (T * V * 2 / 1e9))
    chosen = [0, B - 1]                                           # one fresh sample, one very stale one
    cu0 = orc.segment_offsets(w["seq_lens_host"])
    saved = {i: w["logits"][int(cu0[i]):int(cu0[i + 1])].clone() for i in chosen}
    st = _pass_for(w, alloc_dlogits=False)
    st.token_logprobs(w)
    st.freshness_score(w, HP)
    _sync_ok(st)
    cu = _integers_everywhere(w, st)
    lp = _pass_for(w, alloc_dlogits=False)
    lp.loss_fwd_bwd(w, HP, dlogits=w["logits"])
    _sync_ok(lp)
    assert torch.equal(st.logp, lp.logp) and torch.equal(st.freshness, lp.freshness)
    for i in chosen:
        o = _oracle_sample(w, i, cu, HP, B, logits=saved[i], block=1024)
        # heavy tails: most sampled tokens have p_y within 1e-13 of 1, where z_y - lse cancels in float64;
        # compare log-probs with an absolute tolerance only (the relative check is in test_extreme_rows)
        _check_sample(o, i, lp.logp, st.lse, lp.freshness, lp.weights, st)
        picks = np.unique(np.linspace(0, o["b"] - o["a"] - 1, 5).astype(int))
        _check_sample_grad_rows(o, i, w, lambda rows_: w["logits"][torch.from_numpy(rows_).to(DEV)], picks,
                                logits=saved[i])
        _say("sample %d ok (lag %d, f=%.6f, w=%.6f)" % (i, w["lag_host"][i], o["f"][0], o["w"][0]))
    assert float(lp.weights[0]) > 0.0 and float(lp.weights[B - 1]) == 0.0
    _row_properties(w, cu, lambda t: w["logits"][t], lp.weights, n_rows=32, expect_nonzero=False)
    w_gpu = np64(lp.weights)
    Ls = float(np.sum(w_gpu * (np64(st.ell) + HP[3] * np64(st.D_roll))) / B)
    assert abs(float(lp.loss) - Ls) <= 2e-6 * abs(Ls)


def test_full_vocabulary_drift_variant_at_full_size():
    _say("full-vocabulary KL variant at full size (reasoning + stale logits, 3 x 49.8 GB): generating ...")
    w = wl.generate("reasoning", DEV, seed=0, stale_logit_sigma=0.03)
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]
    hp = HP
    lp = _pass_for(w)
    kl = torch.empty(T, device=DEV)
    fb.fopd_loss_fwd_bwd_full_kl(w["logits"], w["logits_stale"], lp.dt, T, V, ld, ld, w["token_ids"], w["mask"],
                                 w["teacher_logp"], None, w["seq_lens"], w["lag"], B, hp,
                                 None, None, None, 0, None, None, None, None, 1.0, lp.loss, lp.freshness,
                                 lp.weights, lp.logp, kl, lp.dlogits, lp.workspace)
    _sync_ok(lp)
    seq, lag = w["seq_lens_host"], w["lag_host"]
    cu = orc.segment_offsets(seq)
    stale_ones = [i for i in np.argsort(seq, kind="stable") if lag[i] > 0][:2]
    fresh_one = [i for i in np.argsort(seq, kind="stable") if lag[i] == 0][:1]
    f_gpu, w_gpu = np64(lp.freshness), np64(lp.weights)
    for i in [int(x) for x in stale_ones + fresh_one]:
        a, b = int(cu[i]), int(cu[i + 1])
        z, zs = np64(w["logits"][a:b]), np64(w["logits_stale"][a:b])
        y = np64(w["token_ids"][a:b])
        ref = orc.fopd_loss_fwd_bwd_full_kl(z, zs, y, None, np64(w["teacher_logp"][a:b]), None, seq[i:i + 1],
                                            lag[i:i + 1], hp[0], hp[1], hp[2], hp[3], 1.0 / B, want_dlogits=False)
        # (one sample passed alone: its 1/B normaliser is restored through grad_scale = 1/B above)
        assert_close("roll_kl s%d" % i, np64(kl[a:b]), ref["roll_kl"], rtol=2e-5, atol=KL_ROW_ATOL)
        assert_close("logp s%d" % i, np64(lp.logp[a:b]), ref["logp"], atol=1e-4)
        f = ref["freshness"][0]
        assert abs(f_gpu[i] - f) <= 1e-5 * f and abs(w_gpu[i] - ref["weights"][0]) <= 1e-5 * f
        if lag[i] == 0:
            assert not bool(kl[a:b].any()) and abs(f_gpu[i] - 1.0) < 1e-12
        picks = np.unique(np.linspace(0, b - a - 1, 4).astype(int))
        got = np64(lp.dlogits[a:b][torch.from_numpy(picks).to(DEV)])
        check_grad_rows_full_kl(got, z[picks], zs[picks], y[picks], ref, picks, hp, 1.0, B,
                                np.zeros(b - a, dtype=int), "bf16")
        _say("sample %d ok (lag %d, D_roll=%.3e, f=%.6f)" % (i, lag[i], ref["D_roll"][0], f))
    _row_properties(w, cu, lambda t: lp.dlogits[t], lp.weights, n_rows=24)


# ---------------------------------------------------------------------------------------
# the projection in front of the pass: log-probs from hidden states, logits never stored
# ---------------------------------------------------------------------------------------

def _lm_head_call(w, mask=True):
    T = w["T"]
    nbytes = fb.fopd_lm_head_workspace_bytes(T)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=DEV)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + nbytes]
    fb.fopd_workspace_init(ws)
    logp = torch.full((T,), 7.0, dtype=torch.float32, device=DEV)
    lse = torch.full((T,), 7.0, dtype=torch.float32, device=DEV)
    fb.fopd_lm_head_token_logprobs(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, w["V"], w["d"],
                                   w["token_ids"], w["mask"] if mask else None, logp, lse, ws)
    return logp, lse, ws


LM_HEAD_CASES = {
    # T, d, V, ldh, ldw, masked_every: ragged token and vocabulary tiles, strips with no tile, one row
    "ragged_tiles": (300, 128, 1000, 136, 128, 7),
    "one_row_tiny_vocab": (1, 64, 5, 64, 72, 0),
    "exact_tiles": (512, 192, 2048, 192, 192, 0),
    "many_vocab_tiles": (520, 256, 151936, 256, 256, 5),
}


@pytest.mark.gpu
def test_projection_fused_replay_from_a_hip_graph():
    """After one eager call (which sets the kernel's LDS attribute) the entry point enqueues two kernels and
    nothing else, so it can be captured; replays with eager work in between reproduce the eager bits."""
    w = wl.generate_lm_head(600, 128, 5000, DEV, seed=9, masked_every=11)
    logp_e, lse_e, ws = _lm_head_call(w)
    torch.cuda.synchronize()
    logp = torch.zeros_like(logp_e)
    lse = torch.zeros_like(lse_e)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        fb.fopd_lm_head_token_logprobs(w["hidden"], w["ldh"], w["weight"], w["ldw"], w["T"], w["V"], w["d"],
                                       w["token_ids"], w["mask"], logp, lse, ws)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        logp.fill_(float(rep))
        lse.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(logp, logp_e) and torch.equal(lse, lse_e)
    assert fb.fopd_workspace_status(ws) == (0, 0)
    # the number of unmasked rows is read on the device: the captured call follows a mask that changes behind it
    rs = np.random.RandomState(2)
    for m in (rs.choice([0, 1], size=w["T"]).astype(np.uint8), np.ones(w["T"], dtype=np.uint8),
              np.zeros(w["T"], dtype=np.uint8)):
        w["mask"].copy_(torch.from_numpy(m).to(DEV))
        logp_m, lse_m, ws_m = _lm_head_call(w)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(logp, logp_m) and torch.equal(lse, lse_m)
        assert int((lse != 0).sum()) == int(m.sum()) and fb.fopd_workspace_status(ws_m) == (0, 0)


@pytest.mark.gpu
def test_projection_fused_wide_logits():
    """Logits with a spread of 40 (row maxima around 150): the running reference rises by tens between
    vocabulary tiles, so every rescale path of the on-the-fly log-sum-exp is taken."""
    T, d, V = 300, 128, 3000
    w = wl.generate_lm_head(T, d, V, DEV, seed=8, logit_sigma=40.0)
    logp, lse, ws = _lm_head_call(w)
    assert fb.fopd_workspace_status(ws) == (0, 0)
    ref_lse, ref_lp = orc.lm_head_token_logprobs(np64(w["hidden"]), np64(w["weight"]), np64(w["token_ids"]), None)
    # fp32 accumulation of d products: error on a logit of magnitude 150 is a few 1e-5
    assert_close("lse (wide)", np64(lse), ref_lse, rtol=2e-6, atol=1e-4)
    assert_close("logp (wide)", np64(logp), ref_lp, rtol=2e-6, atol=2e-4)


@pytest.mark.gpu
@pytest.mark.parametrize("name", sorted(LM_HEAD_CASES))
def test_projection_fused_logprobs(name):
    T, d, V, ldh, ldw, every = LM_HEAD_CASES[name]
    _say("lm_head %s T=%d d=%d V=%d" % (name, T, d, V))
    w = wl.generate_lm_head(T, d, V, DEV, seed=5, masked_every=every, ldh=ldh, ldw=ldw)
    logp, lse, ws = _lm_head_call(w)
    assert fb.fopd_workspace_status(ws) == (0, 0)
    mask = np64(w["mask"])
    ref_lse, ref_lp = orc.lm_head_token_logprobs(np64(w["hidden"])[:, :d], np64(w["weight"])[:, :d],
                                                 np64(w["token_ids"]), mask)
    # fp32 accumulation over d products of magnitude ~ 3 / sqrt(d): a few 1e-6 on a logit
    assert_close("lse (projection)", np64(lse), ref_lse, rtol=0, atol=1e-4)
    assert_close("logp (projection)", np64(logp), ref_lp, rtol=0, atol=1e-4)
    assert np.all(np64(logp) <= 0.0)
    dead = mask == 0
    assert np.all(np64(logp)[dead] == 0.0) and np.all(np64(lse)[dead] == 0.0)
    # bit-reproducible
    logp2, lse2, _ = _lm_head_call(w)
    assert torch.equal(logp, logp2) and torch.equal(lse, lse2)


@pytest.mark.gpu
def test_projection_fused_leaves_masked_spans_out():
    """Long masked spans (observation turns): only the other rows are projected, gathered through a row map, with
    their count kept on the device.  Against the oracle, and bit for bit against the call that projects every row
    (a token's sums do not depend on where its row sits in a tile); then with every row masked."""
    T, d, V = 2600, 64, 3000
    _say("lm_head with masked spans: T=%d d=%d V=%d" % (T, d, V))
    w = wl.generate_lm_head(T, d, V, DEV, seed=15)
    m = np.ones(T, dtype=np.uint8)
    for a, b in ((0, 300), (700, 1500), (1501, 1800), (2590, 2600)):
        m[a:b] = 0
    w["mask"] = torch.from_numpy(m).to(DEV)
    logp, lse, ws = _lm_head_call(w)
    assert fb.fopd_workspace_status(ws) == (0, 0)
    ref_lse, ref_lp = orc.lm_head_token_logprobs(np64(w["hidden"]), np64(w["weight"]), np64(w["token_ids"]), np64(w["mask"]))
    assert_close("lse (masked spans)", np64(lse), ref_lse, rtol=0, atol=1e-4)
    assert_close("logp (masked spans)", np64(logp), ref_lp, rtol=0, atol=1e-4)
    assert not bool(logp[torch.from_numpy(m == 0).to(DEV)].any()) and bool((lse[torch.from_numpy(m != 0).to(DEV)] != 0).all())
    try:
        fb.fopd_set_option("lm_head_compact", 0)
        logp_all, lse_all, _ = _lm_head_call(w)
    finally:
        fb.fopd_set_option("lm_head_compact", 1)
    assert torch.equal(logp, logp_all) and torch.equal(lse, lse_all)
    w["mask"].zero_()
    logp0, lse0, ws0 = _lm_head_call(w)
    assert fb.fopd_workspace_status(ws0) == (0, 0)
    assert not bool(logp0.any()) and not bool(lse0.any())


@pytest.mark.gpu
def test_projection_fused_more_rows_than_32_bit_offsets_reach():
    """T * ldh beyond 2^31 (a wide row pitch stands in for a long buffer): the call goes through the rows in blocks.
    Rows on both sides of the block boundary, the first and the last against the oracle; masked rows give zeros."""
    d, V, ldh = 64, 500, 8192
    T = (2 ** 31 - 1) // ldh // 256 * 256 + 777                  # one full block of 261,888 rows and a ragged second one
    _say("lm_head in row blocks: T=%d ldh=%d (T * ldh = %.3f * 2^31)" % (T, ldh, T * ldh / 2.0 ** 31))
    gen = torch.Generator(device=DEV)
    gen.manual_seed(77)
    hidden = torch.zeros(T, ldh, dtype=torch.bfloat16, device=DEV)
    hidden[:, :d] = torch.randn(T, d, generator=gen, device=DEV).to(torch.bfloat16)
    weight = (torch.randn(V, d, generator=gen, device=DEV) * 0.4).to(torch.bfloat16)
    token_ids = torch.randint(0, V, (T,), generator=gen, device=DEV, dtype=torch.int32)
    mask = torch.ones(T, dtype=torch.uint8, device=DEV)
    mask[5::7] = 0
    w = dict(T=T, d=d, V=V, ldh=ldh, ldw=d, hidden=hidden, weight=weight, token_ids=token_ids, mask=mask)
    logp, lse, ws = _lm_head_call(w)
    assert fb.fopd_workspace_status(ws) == (0, 0)
    edge = T - 777
    rows = [0, 1, 5, edge - 2, edge - 1, edge, edge + 1, T - 2, T - 1] + [int(x) for x in
                                                                        np.random.RandomState(1).randint(0, T, size=12)]
    idx = torch.tensor(rows, device=DEV)
    ref_lse, ref_lp = orc.lm_head_token_logprobs(np64(hidden[idx, :d]), np64(weight), np64(token_ids[idx]), np64(mask[idx]))
    assert_close("lse (row blocks)", np64(lse[idx]), ref_lse, rtol=0, atol=1e-4)
    assert_close("logp (row blocks)", np64(logp[idx]), ref_lp, rtol=0, atol=1e-4)
    assert not bool(logp[5::7].any()) and not bool(lse[5::7].any())
    assert int((lse != 0).sum()) == int(mask.sum())


@pytest.mark.gpu
def test_projection_fused_token_range_flag_and_empty_call():
    w = wl.generate_lm_head(40, 64, 300, DEV, seed=6)
    w["token_ids"][3] = 300
    w["token_ids"][9] = -1
    logp, lse, ws = _lm_head_call(w)
    assert fb.fopd_workspace_status(ws) == (6, 1)
    assert float(logp[3]) == 0.0 and float(lse[9]) == 0.0 and float(lse[4]) != 0.0
    # no rows: a valid call that touches nothing
    fb.fopd_workspace_init(ws)
    before = logp.clone()
    fb.fopd_lm_head_token_logprobs(w["hidden"], w["ldh"], w["weight"], w["ldw"], 0, w["V"], w["d"],
                                   w["token_ids"], None, logp, lse, ws)
    assert fb.fopd_workspace_status(ws) == (0, 0) and torch.equal(logp, before)


@pytest.mark.gpu
def test_projection_fused_at_benchmark_size_sampled_rows():
    """The projection benchmark's own configuration (rows and mask of the reasoning workload, d = 4096,
    V = 151,936), checked on sampled rows that the oracle computes one by one."""
    seq_lens, mask_host = wl.structure_only("reasoning", seed=0)
    T, d, V = int(seq_lens.sum()), 4096, 151936
    _say("lm_head full size T=%d d=%d V=%d" % (T, d, V))
    w = wl.generate_lm_head(T, d, V, DEV, seed=0)
    mask_host = mask_host.copy()
    mask_host[::97] = 0
    w["mask"] = torch.from_numpy(mask_host).to(DEV)
    logp, lse, ws = _lm_head_call(w)
    assert fb.fopd_workspace_status(ws) == (0, 0)
    rows = [0, 1, 255, 256, 4095, 16384, 100000, T - 257, T - 2, T - 1]
    W64 = w["weight"].float().cpu().numpy().astype(np.float64)
    for t in rows:
        ref_lse, ref_lp = orc.lm_head_token_logprobs(np64(w["hidden"][t:t + 1]), W64, np64(w["token_ids"][t:t + 1]),
                                                     mask_host[t:t + 1])
        assert abs(float(lse[t]) - ref_lse[0]) <= 1e-4, (t, float(lse[t]), ref_lse[0])
        assert abs(float(logp[t]) - ref_lp[0]) <= 1e-4, (t, float(logp[t]), ref_lp[0])
    got = np64(logp)
    assert np.all(got[mask_host == 0] == 0.0) and np.all(got[mask_host != 0] < 0.0)
    assert np.all(np.isfinite(np64(lse)))
    # the same rows through the 8-strip launch shape (a row count that fills the chip exactly)
    T8 = 32768
    w8 = dict(w, T=T8, hidden=w["hidden"][:T8], token_ids=w["token_ids"][:T8], mask=w["mask"][:T8])
    logp8, lse8, ws8 = _lm_head_call(w8)
    assert fb.fopd_workspace_status(ws8) == (0, 0)
    # both launches sum 151,936 fp32 terms per row, in different orders
    assert_close("lse, 8 strips vs 32", np64(lse8), np64(lse)[:T8], rtol=0, atol=1e-4)
    assert_close("logp, 8 strips vs 32", np64(logp8), got[:T8], rtol=0, atol=1e-4)


# ---------------------------------------------------------------------------------------
# the two aligned sets kept apart (mask bytes 0 / 1 / 2 / 3)
# ---------------------------------------------------------------------------------------

def _two_set_workload(seed, **kw):
    w = wl.generate("coding", DEV, seed=seed, B=6, total_len=96, resp_lo=8, resp_hi=24, obs_lo=3, obs_hi=9,
                    aligned_split=(0.3, 0.25), **kw)
    m = w["mask_host"].copy()
    m[96:192][m[96:192] != 0] = 3                 # sample 1: U^roll empty -> invalid
    m[192:288][m[192:288] != 0] = 2               # sample 2: U^sup empty  -> invalid
    m[288] = 200                                  # any other non-zero byte counts as "both"
    w["mask_host"] = m
    w["mask"] = torch.from_numpy(m).to(DEV)
    return w


@pytest.mark.gpu
@pytest.mark.parametrize("V,ld", [(4099, 4104), (151936, 151936)])
def test_two_aligned_sets_all_outputs(V, ld):
    _say("two aligned sets V=%d" % V)
    w = _two_set_workload(31, V=V, ld=ld)
    assert set(np.unique(w["mask_host"])) >= {0, 1, 2, 3}
    hp = (1.0, 1.0, 0.02, 0.4)
    ref, lp = _compare_everything(w, hp, grad_scale=1.5, staged=True)
    assert ref["freshness"][1] == 0.0 and ref["freshness"][2] == 0.0 and ref["agg"][1] != ref["agg"][2]
    # invalid samples stay out whatever the threshold is
    ref2, lp2 = _compare_everything(w, (1.0, 1.0, -0.5, 0.4), grad_scale=1.0, staged=False)
    assert float(lp2.weights[1]) == 0.0 and float(lp2.weights[2]) == 0.0 and float(lp2.weights[0]) > 0.5


@pytest.mark.gpu
def test_two_aligned_sets_scored_and_chunked_flow():
    """Scores supplied (both passes in one kernel) and the chunked gradient with both count arrays passed
    in must give the bits of the all-in-one call."""
    w = _two_set_workload(32, V=9001, ld=9008)
    T, V, B = w["T"], w["V"], w["B"]
    hp = (1.0, 1.0, 0.02, 0.4)
    one = _pass_for(w)
    one.loss_fwd_bwd(w, hp, 0.5)
    st = _pass_for(w, alloc_dlogits=False)
    st.token_logprobs(w)
    st.freshness_score(w, hp)
    _sync_ok(st)
    sc = _pass_for(w)
    fb.fopd_loss_fwd_bwd(w["logits"], sc.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                         w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp,
                         st.freshness, None, None, 0, None, None, 0.5, sc.loss, None, sc.weights, sc.logp,
                         sc.dlogits, sc.workspace)
    _sync_ok(sc)
    # the all-in-one call keeps f_i in fp64, this one reads the fp32 copy: equal to one bf16 ulp, not bitwise
    a64, b64 = np64(sc.dlogits)[:, :V], np64(one.dlogits)[:, :V]
    assert np.all(np.abs(a64 - b64) <= 2.0 ** -7 * np.abs(b64) + 2.0 ** -126)
    assert_close("weights (scored vs fused)", np64(sc.weights), np64(one.weights), rtol=1e-6, atol=1e-9)
    assert abs(float(sc.loss) - float(one.loss)) <= 2e-6 * abs(float(one.loss))
    ck = _pass_for(w)
    ck.dlogits.fill_(3.0)
    tot = 0.0
    for a in range(0, T, 80):                     # chunks cut samples (96 rows each)
        b = min(a + 80, T)
        part = torch.zeros(1, device=DEV)
        fb.fopd_loss_fwd_bwd(w["logits"][a:b], ck.dt, b - a, V, w["ld"], w["token_ids"][a:b], w["mask"][a:b],
                             w["behav_logp"][a:b], w["teacher_logp"][a:b], w["teacher_logp_stale"][a:b],
                             w["seq_lens"], w["lag"], B, hp, st.freshness, st.n_train, st.n_roll, a, st.lse[a:b],
                             st.logp[a:b], 0.5, part, None, ck.weights, None, ck.dlogits[a:b], ck.workspace)
        tot += float(part)
    _sync_ok(ck)
    assert torch.equal(ck.dlogits[:, :V], sc.dlogits[:, :V])       # same bits; padding columns are never written
    assert torch.equal(ck.weights, sc.weights)
    assert abs(tot - float(one.loss)) <= 2e-6 * abs(float(one.loss))


@pytest.mark.gpu
def test_two_aligned_sets_in_the_two_tensor_variants():
    w = _two_set_workload(33, V=5003, ld=5008, stale_logit_sigma=0.05)
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]
    hp = (1.0, 1.0, 0.02, 0.4)
    z, z2 = np64(w["logits"])[:, :V], np64(w["logits_stale"])[:, :V]
    sample_of = np.repeat(np.arange(B), np64(w["seq_lens"]))
    for teacher in (False, True):
        lp = _pass_for(w)
        kl = torch.empty(T, device=DEV)
        if teacher:
            ref = orc.fopd_loss_fwd_bwd_full_teacher(z, z2, np64(w["token_ids"]), np64(w["mask"]), np64(w["behav_logp"]),
                                                     np64(w["teacher_logp"]), np64(w["seq_lens"]), np64(w["lag"]),
                                                     hp[0], hp[1], hp[2], hp[3], 1.2, out_dtype=w["dtype"])
            fb.fopd_loss_fwd_bwd_full_teacher(w["logits"], w["logits_stale"], lp.dt, T, V, ld, ld, w["token_ids"],
                                              w["mask"], w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"],
                                              B, hp, None, None, None, 0, None, None, None, None, 1.2, lp.loss, lp.freshness, lp.weights, lp.logp, kl,
                                              lp.dlogits,
                                              lp.workspace)
        else:
            ref = orc.fopd_loss_fwd_bwd_full_kl(z, z2, np64(w["token_ids"]), np64(w["mask"]), np64(w["teacher_logp"]),
                                                np64(w["teacher_logp_stale"]), np64(w["seq_lens"]), np64(w["lag"]),
                                                hp[0], hp[1], hp[2], hp[3], 1.2, out_dtype=w["dtype"])
            fb.fopd_loss_fwd_bwd_full_kl(w["logits"], w["logits_stale"], lp.dt, T, V, ld, ld, w["token_ids"], w["mask"],
                                         w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp,
                                         None, None, None, 0, None, None, None, None, 1.2, lp.loss, lp.freshness, lp.weights, lp.logp, kl, lp.dlogits, lp.workspace)
        _sync_ok(lp)
        assert_close("freshness", np64(lp.freshness), ref["freshness"], rtol=1e-5)
        assert_close("weights", np64(lp.weights), ref["weights"], atol=1e-5 * ref["freshness"] + 1e-12)
        assert abs(float(lp.loss) - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-12
        assert ref["freshness"][1] == 0.0 and ref["freshness"][2] == 0.0
        ref.setdefault("delta", np.zeros(T))
        ref.setdefault("rho", np.ones(T))
        check_grad_rows_full_kl(np64(lp.dlogits)[:, :V], z, z2, np64(w["token_ids"]), ref, range(T), hp, 1.2, B,
                                sample_of, w["dtype"], c2_scales_with_weight=teacher)
