"""ctypes binding of include/fopd.h.

Argument marshalling only: every function here has the name and argument order of the C entry
point it calls, takes torch tensors (or raw device addresses as ints) for the pointer
arguments, and launches on torch's current stream unless told otherwise.  All arithmetic runs
in the HIP kernels; if the shared library is missing or cannot be loaded this module raises.
"""

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "lib", "libfopd.so")

FOPD_F32 = 0
FOPD_BF16 = 1

SYMBOLS = (
    "fopd_status_string", "fopd_workspace_bytes", "fopd_workspace_init", "fopd_workspace_status", "fopd_flags_status",
    "fopd_token_logprobs", "fopd_freshness_score", "fopd_loss_fwd_bwd", "fopd_loss_fwd_bwd_unit", "fopd_loss_fwd_bwd_static",
    "fopd_profile_enable", "fopd_profile_reset", "fopd_profile_read", "fopd_set_option",
    "fopd_refresh_decide", "fopd_rollout_kl", "fopd_loss_fwd_bwd_full_kl", "fopd_loss_fwd_bwd_full_teacher",
    "fopd_topk_workspace_bytes", "fopd_topk_token_loss", "fopd_loss_fwd_bwd_topk_teacher",
    "fopd_lm_head_workspace_bytes", "fopd_lm_head_token_logprobs",
    "fopd_lm_head_loss_workspace_bytes", "fopd_lm_head_loss_fwd_bwd",
    "fopd_lm_head_loss_topk_workspace_bytes", "fopd_lm_head_loss_fwd_bwd_topk_teacher",
)


class Hparams(ctypes.Structure):
    """fopd_hparams: alpha, beta (score coefficients), xi (gate), lambda (anchor strength)."""
    _fields_ = [("alpha", ctypes.c_float), ("beta", ctypes.c_float),
                ("xi", ctypes.c_float), ("lambda_", ctypes.c_float)]


class RefreshConfig(ctypes.Structure):
    """fopd_refresh_config: thresholds kappa_f, kappa_roll, kappa_sup and the rate limit in steps."""
    _fields_ = [("kappa_f", ctypes.c_float), ("kappa_roll", ctypes.c_float), ("kappa_sup", ctypes.c_float),
                ("min_interval", ctypes.c_int64)]


class RefreshState(ctypes.Structure):
    _fields_ = [("last_refresh_step", ctypes.c_int64), ("refreshes", ctypes.c_int64)]

    def __init__(self):
        super().__init__(-1, 0)


class FopdError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: status %d (%s)" % (where, self.status, fopd_status_string(self.status)))


_lib = None


def library_path():
    return _LIB_PATH


def load_library():
    """Loads lib/libfopd.so (built by paper_2605_17862_amd/build.py).  Fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("HIP library not built: %s is missing (run `python -m paper_2605_17862_amd.build`)"
                          % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    lib.fopd_status_string.restype = ctypes.c_char_p
    lib.fopd_status_string.argtypes = [ctypes.c_int]
    lib.fopd_workspace_bytes.restype = sz
    lib.fopd_workspace_bytes.argtypes = [i64, i32]
    lib.fopd_workspace_init.restype = ctypes.c_int
    lib.fopd_workspace_init.argtypes = [vp, sz, vp]
    lib.fopd_workspace_status.restype = ctypes.c_int
    lib.fopd_workspace_status.argtypes = [vp, vp, ctypes.POINTER(i32)]
    lib.fopd_flags_status.restype = ctypes.c_int
    lib.fopd_flags_status.argtypes = [i32]
    lib.fopd_token_logprobs.restype = ctypes.c_int
    lib.fopd_token_logprobs.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fopd_lm_head_workspace_bytes.restype = sz
    lib.fopd_lm_head_workspace_bytes.argtypes = [i64]
    lib.fopd_lm_head_token_logprobs.restype = ctypes.c_int
    lib.fopd_lm_head_token_logprobs.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.fopd_lm_head_loss_workspace_bytes.restype = sz
    lib.fopd_lm_head_loss_workspace_bytes.argtypes = [i64, i64, i64, i32, i64]
    lib.fopd_lm_head_loss_fwd_bwd.restype = ctypes.c_int
    lib.fopd_lm_head_loss_fwd_bwd.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, i32, Hparams,
                                              vp, vp, vp, vp, f32, i64, vp, vp, vp, vp, vp, vp, i64, vp, i64,
                                              ctypes.c_int, vp, sz, vp]
    lib.fopd_lm_head_loss_topk_workspace_bytes.restype = sz
    lib.fopd_lm_head_loss_topk_workspace_bytes.argtypes = [i64, i64, i64, i32, i64, i32]
    lib.fopd_lm_head_loss_fwd_bwd_topk_teacher.restype = ctypes.c_int
    lib.fopd_lm_head_loss_fwd_bwd_topk_teacher.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, vp, vp, vp, vp, i32, f32,
                                                           vp, vp, vp, vp, i32, Hparams, vp, vp, vp, vp, f32, i64, vp, vp,
                                                           vp, vp, vp, vp, vp, i64, vp, i64, ctypes.c_int, vp, sz, vp]
    lib.fopd_freshness_score.restype = ctypes.c_int
    lib.fopd_freshness_score.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, Hparams,
                                         vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fopd_rollout_kl.restype = ctypes.c_int
    lib.fopd_rollout_kl.argtypes = [vp, vp, ctypes.c_int, i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fopd_loss_fwd_bwd_full_teacher.restype = ctypes.c_int
    lib.fopd_loss_fwd_bwd_full_teacher.argtypes = [vp, vp, ctypes.c_int, i64, i64, i64, i64, vp, vp, vp, vp, vp, vp,
                                                   i32, Hparams, vp, vp, vp, i64, vp, vp, vp, vp, f32,
                                                   vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fopd_topk_workspace_bytes.restype = sz
    lib.fopd_topk_workspace_bytes.argtypes = [i64, i32, i32]
    lib.fopd_loss_fwd_bwd_topk_teacher.restype = ctypes.c_int
    lib.fopd_loss_fwd_bwd_topk_teacher.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp, vp, i32, f32, vp, vp,
                                                   vp, vp, i32, Hparams, vp, vp, vp, i64, vp, vp, f32, vp, vp, vp, vp,
                                                   vp, vp, vp, sz, vp]
    lib.fopd_topk_token_loss.restype = ctypes.c_int
    lib.fopd_topk_token_loss.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp, i32, f32, vp, vp, vp]
    lib.fopd_loss_fwd_bwd_full_kl.restype = ctypes.c_int
    lib.fopd_loss_fwd_bwd_full_kl.argtypes = [vp, vp, ctypes.c_int, i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, i32,
                                              Hparams, vp, vp, vp, i64, vp, vp, vp, vp, f32,
                                              vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fopd_loss_fwd_bwd.restype = ctypes.c_int
    lib.fopd_loss_fwd_bwd.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, i32, Hparams,
                                      vp, vp, vp, i64, vp, vp, f32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fopd_loss_fwd_bwd_unit.restype = ctypes.c_int
    lib.fopd_loss_fwd_bwd_unit.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, i32, Hparams,
                                           f32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fopd_loss_fwd_bwd_static.restype = ctypes.c_int
    lib.fopd_loss_fwd_bwd_static.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, i32, Hparams,
                                             vp, vp, vp, i64, vp, vp, f32, vp, vp, vp, vp, vp, vp, vp]
    lib.fopd_refresh_decide.restype = ctypes.c_int
    lib.fopd_refresh_decide.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(RefreshConfig),
                                        ctypes.POINTER(RefreshState), i64, ctypes.POINTER(i32)]
    lib.fopd_set_option.restype = ctypes.c_int
    lib.fopd_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int]
    lib.fopd_profile_enable.restype = ctypes.c_int
    lib.fopd_profile_enable.argtypes = [ctypes.c_int]
    lib.fopd_profile_reset.restype = ctypes.c_int
    lib.fopd_profile_reset.argtypes = []
    lib.fopd_profile_read.restype = ctypes.c_int
    lib.fopd_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    _lib = lib
    return lib


def _ptr(x, dtype=None, name="argument"):
    """Device address of a tensor (checked: contiguous, on a GPU, expected dtype), an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    if not x.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if not x.is_cuda:
        raise ValueError("%s must live in device memory" % name)
    if dtype is not None and x.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise ValueError("%s has dtype %s, expected %s" % (name, x.dtype, dtype))
    return ctypes.c_void_p(x.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return ctypes.c_void_p(int(stream))


def _check(status, where):
    if status != 0:
        raise FopdError(status, where)


def _hp(hp):
    if isinstance(hp, Hparams):
        return hp
    alpha, beta, xi, lam = hp
    return Hparams(float(alpha), float(beta), float(xi), float(lam))


def _ws(workspace):
    if isinstance(workspace, tuple):
        return ctypes.c_void_p(int(workspace[0])), int(workspace[1])
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def fopd_status_string(status):
    return load_library().fopd_status_string(int(status)).decode()


def fopd_workspace_bytes(T, B):
    return int(load_library().fopd_workspace_bytes(int(T), int(B)))


def fopd_workspace_init(workspace, stream=None):
    p, n = _ws(workspace)
    _check(load_library().fopd_workspace_init(p, n, _stream(stream)), "fopd_workspace_init")


def fopd_workspace_status(workspace, stream=None):
    """Host-synchronous.  Returns (status, flag bits)."""
    p, _ = _ws(workspace)
    flags = ctypes.c_int32(0)
    st = load_library().fopd_workspace_status(p, _stream(stream), ctypes.byref(flags))
    return int(st), int(flags.value)


def fopd_token_logprobs(logits, dt, T, V, ld, token_ids, mask, logp, lse, gather_idx, entropy, workspace,
                        stream=None):
    import torch
    p, n = _ws(workspace)
    st = load_library().fopd_token_logprobs(
        _ptr(logits, (torch.float32, torch.bfloat16), "logits"), int(dt), int(T), int(V), int(ld),
        _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(logp, torch.float32, "logp"), _ptr(lse, torch.float32, "lse"),
        _ptr(gather_idx, torch.int64, "gather_idx"), _ptr(entropy, torch.float32, "entropy"),
        p, n, _stream(stream))
    _check(st, "fopd_token_logprobs")


def fopd_lm_head_workspace_bytes(T):
    return int(load_library().fopd_lm_head_workspace_bytes(int(T)))


def fopd_lm_head_token_logprobs(hidden, ldh, weight, ldw, T, V, d, token_ids, mask, logp, lse, workspace,
                                stream=None):
    import torch
    p, n = _ws(workspace)
    st = load_library().fopd_lm_head_token_logprobs(
        _ptr(hidden, torch.bfloat16, "hidden"), int(ldh), _ptr(weight, torch.bfloat16, "weight"), int(ldw),
        int(T), int(V), int(d), _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(logp, torch.float32, "logp"), _ptr(lse, torch.float32, "lse"), p, n, _stream(stream))
    _check(st, "fopd_lm_head_token_logprobs")


def fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk):
    return int(load_library().fopd_lm_head_loss_workspace_bytes(int(T), int(V), int(d), int(B), int(rows_chunk)))


def fopd_lm_head_loss_fwd_bwd(hidden, ldh, weight, ldw, T, V, d, token_ids, mask, behav_logp, teacher_logp, seq_lens,
                              lag, B, hp, freshness_in, n_train_in, n_roll_in, grad_scale, rows_chunk, loss, weights,
                              logp, lse, dhidden, lddh, dweight, lddw, accumulate_dweight, workspace, stream=None,
                              seq_lens_host=None, freshness=None):
    """seq_lens_host: the sample lengths in HOST memory (a CPU int32 tensor, a numpy array or a list), needed when
    freshness_in is None (the scores are then formed inside the call); freshness: [B] f32 output or None."""
    import numpy as np
    import torch
    f32 = torch.float32
    p, n = _ws(workspace)
    host = None
    if seq_lens_host is not None:
        if isinstance(seq_lens_host, torch.Tensor):
            if seq_lens_host.is_cuda:
                raise TypeError("seq_lens_host must be in host memory")
            seq_lens_host = seq_lens_host.numpy()
        host = np.ascontiguousarray(np.asarray(seq_lens_host), dtype=np.int32)
        if host.shape != (int(B),):
            raise ValueError("seq_lens_host must hold B lengths")
    st = load_library().fopd_lm_head_loss_fwd_bwd(
        _ptr(hidden, torch.bfloat16, "hidden"), int(ldh), _ptr(weight, torch.bfloat16, "weight"), int(ldw),
        int(T), int(V), int(d), _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(behav_logp, f32, "behav_logp"), _ptr(teacher_logp, f32, "teacher_logp"),
        _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(lag, torch.int32, "lag"), int(B), _hp(hp),
        _ptr(freshness_in, f32, "freshness_in"), _ptr(n_train_in, torch.int32, "n_train_in"),
        _ptr(n_roll_in, torch.int32, "n_roll_in"),
        None if host is None else ctypes.c_void_p(host.ctypes.data), float(grad_scale), int(rows_chunk),
        _ptr(loss, f32, "loss"), _ptr(freshness, f32, "freshness"), _ptr(weights, f32, "weights"),
        _ptr(logp, f32, "logp"), _ptr(lse, f32, "lse"),
        _ptr(dhidden, f32, "dhidden"), int(lddh), _ptr(dweight, f32, "dweight"), int(lddw),
        int(bool(accumulate_dweight)), p, n, _stream(stream))
    _check(st, "fopd_lm_head_loss_fwd_bwd")


def _host_lengths(seq_lens_host, B):
    import numpy as np
    import torch
    if isinstance(seq_lens_host, torch.Tensor):
        if seq_lens_host.is_cuda:
            raise TypeError("seq_lens_host must be in host memory")
        seq_lens_host = seq_lens_host.numpy()
    host = np.ascontiguousarray(np.asarray(seq_lens_host), dtype=np.int32)
    if host.shape != (int(B),):
        raise ValueError("seq_lens_host must hold B lengths")
    return host


def fopd_lm_head_loss_topk_workspace_bytes(T, V, d, B, rows_chunk, k):
    return int(load_library().fopd_lm_head_loss_topk_workspace_bytes(int(T), int(V), int(d), int(B), int(rows_chunk),
                                                                     int(k)))


def fopd_lm_head_loss_fwd_bwd_topk_teacher(hidden, ldh, weight, ldw, T, V, d, token_ids, mask, behav_logp, list_ids,
                                           list_logp, k, rest_floor, teacher_logp, teacher_logp_stale, seq_lens, lag, B,
                                           hp, seq_lens_host, grad_scale, rows_chunk, loss, freshness, weights, logp,
                                           lse, token_loss, dhidden, lddh, dweight, lddw, accumulate_dweight, workspace,
                                           stream=None, freshness_in=None, n_train_in=None, n_roll_in=None):
    """seq_lens_host: the sample lengths in HOST memory (a CPU int32 tensor, a numpy array or a list); not needed
    when freshness_in (scores formed earlier, with n_train_in / n_roll_in from fopd_freshness_score or None) is given."""
    import torch
    f32 = torch.float32
    p, n = _ws(workspace)
    host = None if seq_lens_host is None else _host_lengths(seq_lens_host, B)
    st = load_library().fopd_lm_head_loss_fwd_bwd_topk_teacher(
        _ptr(hidden, torch.bfloat16, "hidden"), int(ldh), _ptr(weight, torch.bfloat16, "weight"), int(ldw),
        int(T), int(V), int(d), _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(behav_logp, f32, "behav_logp"), _ptr(list_ids, torch.int32, "list_ids"), _ptr(list_logp, f32, "list_logp"),
        int(k), float(rest_floor), _ptr(teacher_logp, f32, "teacher_logp"),
        _ptr(teacher_logp_stale, f32, "teacher_logp_stale"), _ptr(seq_lens, torch.int32, "seq_lens"),
        _ptr(lag, torch.int32, "lag"), int(B), _hp(hp), _ptr(freshness_in, f32, "freshness_in"),
        _ptr(n_train_in, torch.int32, "n_train_in"), _ptr(n_roll_in, torch.int32, "n_roll_in"),
        None if host is None else ctypes.c_void_p(host.ctypes.data),
        float(grad_scale), int(rows_chunk), _ptr(loss, f32, "loss"), _ptr(freshness, f32, "freshness"),
        _ptr(weights, f32, "weights"), _ptr(logp, f32, "logp"), _ptr(lse, f32, "lse"),
        _ptr(token_loss, f32, "token_loss"), _ptr(dhidden, f32, "dhidden"), int(lddh), _ptr(dweight, f32, "dweight"),
        int(lddw), int(bool(accumulate_dweight)), p, n, _stream(stream))
    _check(st, "fopd_lm_head_loss_fwd_bwd_topk_teacher")


def fopd_flags_status(flags):
    """Host only: the status code a raw device flag word stands for."""
    return int(load_library().fopd_flags_status(int(flags)))


def fopd_freshness_score(logp, behav_logp, roll_kl, token_loss, teacher_logp, teacher_logp_stale, mask, seq_lens, lag,
                         T, B,
                         hp, cu_seqlens, n_train, n_roll, D_roll, D_sup, ell, cover, cover_roll, freshness, agg,
                         workspace, stream=None):
    import torch
    f32 = torch.float32
    p, n = _ws(workspace)
    st = load_library().fopd_freshness_score(
        _ptr(logp, f32, "logp"), _ptr(behav_logp, f32, "behav_logp"), _ptr(roll_kl, f32, "roll_kl"),
        _ptr(token_loss, f32, "token_loss"), _ptr(teacher_logp, f32, "teacher_logp"),
        _ptr(teacher_logp_stale, f32, "teacher_logp_stale"), _ptr(mask, torch.uint8, "mask"),
        _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(lag, torch.int32, "lag"), int(T), int(B), _hp(hp),
        _ptr(cu_seqlens, torch.int64, "cu_seqlens"), _ptr(n_train, torch.int32, "n_train"),
        _ptr(n_roll, torch.int32, "n_roll"),
        _ptr(D_roll, f32, "D_roll"), _ptr(D_sup, f32, "D_sup"), _ptr(ell, f32, "ell"),
        _ptr(cover, f32, "cover"), _ptr(cover_roll, f32, "cover_roll"), _ptr(freshness, f32, "freshness"),
        _ptr(agg, f32, "agg"),
        p, n, _stream(stream))
    _check(st, "fopd_freshness_score")


def fopd_loss_fwd_bwd(logits, dt, T, V, ld, token_ids, mask, behav_logp, teacher_logp, teacher_logp_stale,
                      seq_lens, lag, B, hp, freshness_in, n_train_in, n_roll_in, row_begin, lse_in, logp_in,
                      grad_scale, loss, freshness, weights, logp, dlogits, workspace, stream=None):
    import torch
    f32 = torch.float32
    mat = (torch.float32, torch.bfloat16)
    p, n = _ws(workspace)
    st = load_library().fopd_loss_fwd_bwd(
        _ptr(logits, mat, "logits"), int(dt), int(T), int(V), int(ld),
        _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(behav_logp, f32, "behav_logp"), _ptr(teacher_logp, f32, "teacher_logp"),
        _ptr(teacher_logp_stale, f32, "teacher_logp_stale"),
        _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(lag, torch.int32, "lag"), int(B), _hp(hp),
        _ptr(freshness_in, f32, "freshness_in"), _ptr(n_train_in, torch.int32, "n_train_in"),
        _ptr(n_roll_in, torch.int32, "n_roll_in"), int(row_begin),
        _ptr(lse_in, f32, "lse_in"), _ptr(logp_in, f32, "logp_in"), float(grad_scale),
        _ptr(loss, f32, "loss"), _ptr(freshness, f32, "freshness"), _ptr(weights, f32, "weights"),
        _ptr(logp, f32, "logp"), _ptr(dlogits, mat, "dlogits"), p, n, _stream(stream))
    _check(st, "fopd_loss_fwd_bwd")


def fopd_loss_fwd_bwd_unit(logits, dt, T, V, ld, token_ids, mask, behav_logp, teacher_logp, teacher_logp_stale,
                           seq_lens, lag, B, hp, grad_scale, loss, freshness, weights, logp, unit_rows, workspace,
                           stream=None):
    import torch
    f32 = torch.float32
    mat = (torch.float32, torch.bfloat16)
    p, n = _ws(workspace)
    st = load_library().fopd_loss_fwd_bwd_unit(
        _ptr(logits, mat, "logits"), int(dt), int(T), int(V), int(ld),
        _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(behav_logp, f32, "behav_logp"), _ptr(teacher_logp, f32, "teacher_logp"),
        _ptr(teacher_logp_stale, f32, "teacher_logp_stale"),
        _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(lag, torch.int32, "lag"), int(B), _hp(hp),
        float(grad_scale), _ptr(loss, f32, "loss"), _ptr(freshness, f32, "freshness"),
        _ptr(weights, f32, "weights"), _ptr(logp, f32, "logp"), _ptr(unit_rows, mat, "unit_rows"), p, n,
        _stream(stream))
    _check(st, "fopd_loss_fwd_bwd_unit")


FOPD_STATIC_MAX_ROWS = 32768
FOPD_STATIC_MAX_SAMPLES = 4096


def fopd_loss_fwd_bwd_static(logits, dt, T, V, ld, token_ids, mask, behav_logp, teacher_logp, teacher_logp_stale,
                             seq_lens, lag, B, hp, freshness_in, n_train_in, n_roll_in, row_begin, lse_in, logp_in,
                             grad_scale, loss, freshness, weights, logp, dlogits, flags_out, stream=None):
    import torch
    f32 = torch.float32
    mat = (torch.float32, torch.bfloat16)
    st = load_library().fopd_loss_fwd_bwd_static(
        _ptr(logits, mat, "logits"), int(dt), int(T), int(V), int(ld),
        _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(behav_logp, f32, "behav_logp"), _ptr(teacher_logp, f32, "teacher_logp"),
        _ptr(teacher_logp_stale, f32, "teacher_logp_stale"),
        _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(lag, torch.int32, "lag"), int(B), _hp(hp),
        _ptr(freshness_in, f32, "freshness_in"), _ptr(n_train_in, torch.int32, "n_train_in"),
        _ptr(n_roll_in, torch.int32, "n_roll_in"), int(row_begin),
        _ptr(lse_in, f32, "lse_in"), _ptr(logp_in, f32, "logp_in"), float(grad_scale),
        _ptr(loss, f32, "loss"), _ptr(freshness, f32, "freshness"), _ptr(weights, f32, "weights"),
        _ptr(logp, f32, "logp"), _ptr(dlogits, mat, "dlogits"), _ptr(flags_out, torch.int32, "flags_out"),
        _stream(stream))
    _check(st, "fopd_loss_fwd_bwd_static")


def fopd_rollout_kl(logits, logits_stale, dt, T, V, ld, ld_stale, token_ids, mask, roll_kl, logp, lse, dlse, logq,
                    workspace, stream=None):
    import torch
    f32 = torch.float32
    mat = (torch.float32, torch.bfloat16)
    p, n = _ws(workspace)
    st = load_library().fopd_rollout_kl(
        _ptr(logits, mat, "logits"), _ptr(logits_stale, mat, "logits_stale"), int(dt), int(T), int(V), int(ld),
        int(ld_stale), _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(roll_kl, f32, "roll_kl"), _ptr(logp, f32, "logp"), _ptr(lse, f32, "lse"), _ptr(dlse, f32, "dlse"),
        _ptr(logq, f32, "logq"), p, n, _stream(stream))
    _check(st, "fopd_rollout_kl")


def fopd_loss_fwd_bwd_full_kl(logits, logits_stale, dt, T, V, ld, ld_stale, token_ids, mask, teacher_logp,
                              teacher_logp_stale, seq_lens, lag, B, hp, freshness_in, n_train_in, n_roll_in, row_begin,
                              lse_in, logp_in, dlse_in, roll_kl_in, grad_scale, loss, freshness, weights, logp,
                              roll_kl, dlogits, workspace, stream=None):
    import torch
    f32 = torch.float32
    mat = (torch.float32, torch.bfloat16)
    p, n = _ws(workspace)
    st = load_library().fopd_loss_fwd_bwd_full_kl(
        _ptr(logits, mat, "logits"), _ptr(logits_stale, mat, "logits_stale"), int(dt), int(T), int(V), int(ld),
        int(ld_stale), _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(teacher_logp, f32, "teacher_logp"), _ptr(teacher_logp_stale, f32, "teacher_logp_stale"),
        _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(lag, torch.int32, "lag"), int(B), _hp(hp),
        _ptr(freshness_in, f32, "freshness_in"), _ptr(n_train_in, torch.int32, "n_train_in"),
        _ptr(n_roll_in, torch.int32, "n_roll_in"), int(row_begin), _ptr(lse_in, f32, "lse_in"),
        _ptr(logp_in, f32, "logp_in"), _ptr(dlse_in, f32, "dlse_in"), _ptr(roll_kl_in, f32, "roll_kl_in"),
        float(grad_scale),
        _ptr(loss, f32, "loss"), _ptr(freshness, f32, "freshness"), _ptr(weights, f32, "weights"),
        _ptr(logp, f32, "logp"), _ptr(roll_kl, f32, "roll_kl"), _ptr(dlogits, mat, "dlogits"), p, n,
        _stream(stream))
    _check(st, "fopd_loss_fwd_bwd_full_kl")


def fopd_loss_fwd_bwd_full_teacher(logits, teacher_logits, dt, T, V, ld, ld_teacher, token_ids, mask, behav_logp,
                                   teacher_logp_stale, seq_lens, lag, B, hp, freshness_in, n_train_in, n_roll_in,
                                   row_begin, lse_in, logp_in, dlse_in, token_kl_in, grad_scale, loss, freshness,
                                   weights, logp, token_kl, dlogits, workspace, stream=None):
    import torch
    f32 = torch.float32
    mat = (torch.float32, torch.bfloat16)
    p, n = _ws(workspace)
    st = load_library().fopd_loss_fwd_bwd_full_teacher(
        _ptr(logits, mat, "logits"), _ptr(teacher_logits, mat, "teacher_logits"), int(dt), int(T), int(V), int(ld),
        int(ld_teacher), _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(behav_logp, f32, "behav_logp"), _ptr(teacher_logp_stale, f32, "teacher_logp_stale"),
        _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(lag, torch.int32, "lag"), int(B), _hp(hp),
        _ptr(freshness_in, f32, "freshness_in"), _ptr(n_train_in, torch.int32, "n_train_in"),
        _ptr(n_roll_in, torch.int32, "n_roll_in"), int(row_begin), _ptr(lse_in, f32, "lse_in"),
        _ptr(logp_in, f32, "logp_in"), _ptr(dlse_in, f32, "dlse_in"), _ptr(token_kl_in, f32, "token_kl_in"),
        float(grad_scale),
        _ptr(loss, f32, "loss"), _ptr(freshness, f32, "freshness"), _ptr(weights, f32, "weights"),
        _ptr(logp, f32, "logp"), _ptr(token_kl, f32, "token_kl"), _ptr(dlogits, mat, "dlogits"), p, n,
        _stream(stream))
    _check(st, "fopd_loss_fwd_bwd_full_teacher")


def fopd_topk_workspace_bytes(T, B, k):
    return int(load_library().fopd_topk_workspace_bytes(int(T), int(B), int(k)))


def fopd_topk_token_loss(logits, dt, T, V, ld, token_ids, mask, list_ids, list_logp, k, rest_floor, lse, token_loss,
                         stream=None):
    import torch
    f32 = torch.float32
    st = load_library().fopd_topk_token_loss(
        _ptr(logits, (torch.float32, torch.bfloat16), "logits"), int(dt), int(T), int(V), int(ld),
        _ptr(token_ids, torch.int32, "token_ids"), _ptr(mask, torch.uint8, "mask"),
        _ptr(list_ids, torch.int32, "list_ids"), _ptr(list_logp, f32, "list_logp"), int(k), float(rest_floor),
        _ptr(lse, f32, "lse"), _ptr(token_loss, f32, "token_loss"), _stream(stream))
    _check(st, "fopd_topk_token_loss")


def fopd_loss_fwd_bwd_topk_teacher(logits, dt, T, V, ld, token_ids, mask, behav_logp, list_ids, list_logp, k,
                                   rest_floor, teacher_logp, teacher_logp_stale, seq_lens, lag, B, hp, freshness_in,
                                   n_train_in, n_roll_in, row_begin, lse_in, logp_in, grad_scale, loss, freshness,
                                   weights, logp, token_loss, dlogits, workspace, stream=None):
    import torch
    f32 = torch.float32
    mat = (torch.float32, torch.bfloat16)
    p, n = _ws(workspace)
    st = load_library().fopd_loss_fwd_bwd_topk_teacher(
        _ptr(logits, mat, "logits"), int(dt), int(T), int(V), int(ld), _ptr(token_ids, torch.int32, "token_ids"),
        _ptr(mask, torch.uint8, "mask"), _ptr(behav_logp, f32, "behav_logp"), _ptr(list_ids, torch.int32, "list_ids"),
        _ptr(list_logp, f32, "list_logp"), int(k), float(rest_floor), _ptr(teacher_logp, f32, "teacher_logp"),
        _ptr(teacher_logp_stale, f32, "teacher_logp_stale"), _ptr(seq_lens, torch.int32, "seq_lens"),
        _ptr(lag, torch.int32, "lag"), int(B), _hp(hp), _ptr(freshness_in, f32, "freshness_in"),
        _ptr(n_train_in, torch.int32, "n_train_in"), _ptr(n_roll_in, torch.int32, "n_roll_in"), int(row_begin),
        _ptr(lse_in, f32, "lse_in"), _ptr(logp_in, f32, "logp_in"), float(grad_scale), _ptr(loss, f32, "loss"),
        _ptr(freshness, f32, "freshness"), _ptr(weights, f32, "weights"), _ptr(logp, f32, "logp"),
        _ptr(token_loss, f32, "token_loss"), _ptr(dlogits, mat, "dlogits"), p, n, _stream(stream))
    _check(st, "fopd_loss_fwd_bwd_topk_teacher")


def fopd_refresh_decide(agg_host, cfg, state, step):
    """Host only.  agg_host: three floats (a host copy of `agg`).  Returns (refresh?, reason bits)."""
    arr = (ctypes.c_float * 3)(*[float(x) for x in agg_host])
    reason = ctypes.c_int32(0)
    r = load_library().fopd_refresh_decide(arr, ctypes.byref(cfg), ctypes.byref(state), int(step),
                                           ctypes.byref(reason))
    if r < 0:
        raise FopdError(1, "fopd_refresh_decide")
    return bool(r), int(reason.value)


def fopd_set_option(name, value):
    _check(load_library().fopd_set_option(name.encode(), int(value)), "fopd_set_option")


def fopd_profile_enable(on):
    _check(load_library().fopd_profile_enable(int(bool(on))), "fopd_profile_enable")


def fopd_profile_reset():
    _check(load_library().fopd_profile_reset(), "fopd_profile_reset")


def fopd_profile_read(which):
    """Host-synchronous.  Returns (total milliseconds, number of launches) of kernel `which`."""
    ms = ctypes.c_double(0.0)
    n = ctypes.c_int64(0)
    _check(load_library().fopd_profile_read(int(which), ctypes.byref(ms), ctypes.byref(n)), "fopd_profile_read")
    return float(ms.value), int(n.value)
