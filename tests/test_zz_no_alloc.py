"""The entry point that allocates nothing (its scratch memory is an array inside the library) against the
entry point it is a variant of, through the C ABI: two calls in a row, the second on a smaller input, every
output compared bit for bit; then the mode whose scores are supplied, the size limits and the device flags."""

import pytest
import torch

from harness import workloads as wl
from paper_2605_17862_amd import binding as fb
from paper_2605_17862_amd.loss_pass import LossPass

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HP = (1.0, 1.0, 0.05, 0.1)


def _both(w, hp, mode="fused", f_in=None, n_in=None):
    """Runs fopd_loss_fwd_bwd (caller's workspace) and fopd_loss_fwd_bwd_static on the same inputs."""
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]
    ref = LossPass(T, V, B, w["dtype"], ld=ld, device=DEV)
    got = LossPass(T, V, B, w["dtype"], ld=ld, device=DEV)
    ref.dlogits.fill_(3.0)
    got.dlogits.fill_(5.0)
    flags = torch.full((1,), 77, dtype=torch.int32, device=DEV)
    common = (w["logits"], ref.dt, T, V, ld, w["token_ids"], w["mask"], w["behav_logp"], w["teacher_logp"],
              w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp, f_in, n_in, None, 0, None, None, 1.5)
    fb.fopd_loss_fwd_bwd(*common, ref.loss, ref.freshness, ref.weights, ref.logp, ref.dlogits, ref.workspace)
    fb.fopd_loss_fwd_bwd_static(*common, got.loss, got.freshness, got.weights, got.logp, got.dlogits, flags)
    torch.cuda.synchronize()
    assert ref.status() == (0, 0)
    assert int(flags) == 0
    assert torch.equal(got.loss, ref.loss) and torch.equal(got.freshness, ref.freshness)
    assert torch.equal(got.weights, ref.weights) and torch.equal(got.logp, ref.logp)
    assert torch.equal(got.dlogits[:, :V], ref.dlogits[:, :V])
    if ld > V:
        assert bool((got.dlogits[:, V:] == 5.0).all())
    assert bool(got.dlogits[:, :V].any())
    return ref


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    print("[no-alloc] first call: tooluse replica, 5 samples, V=9001 bf16", flush=True)
    big = wl.generate("tooluse", DEV, seed=71, B=5, turns=3, obs_lo=2, obs_hi=6, resp_lo=4, resp_hi=20, V=9001, ld=9008,
                      lag_lo=0, lag_hi=30, row_block=64)
    ref = _both(big, HP)
    assert bool((ref.weights == 0).any()) and bool((ref.weights > 0).any())      # gated and live samples
    print("[no-alloc] second call, smaller input: tiny replica, 2 samples, V=640 f32", flush=True)
    small = wl.generate("tiny", DEV, seed=72, B=2, len_lo=9, len_hi=9, V=640)
    _both(small, HP)
    print("[no-alloc] scores supplied (both passes in one kernel), again larger then smaller", flush=True)
    _both(big, HP, f_in=ref.freshness.clone())
    _both(small, HP, f_in=torch.tensor([0.9, 0.01], device=DEV))


def test_static_scratch_entry_point_limits_and_flags():
    w = wl.generate("tiny", DEV, seed=73, B=2, len_lo=6, len_hi=6, V=64)
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]
    lp = LossPass(T, V, B, w["dtype"], ld=ld, device=DEV)
    args = [w["logits"], lp.dt, T, V, ld, w["token_ids"], w["mask"], w["behav_logp"], w["teacher_logp"], None,
            w["seq_lens"], w["lag"], B, HP, None, None, None, 0, None, None, 1.0, lp.loss, lp.freshness, lp.weights,
            lp.logp, lp.dlogits, None]
    too_many_rows = list(args)
    too_many_rows[2] = fb.FOPD_STATIC_MAX_ROWS + 1
    with pytest.raises(fb.FopdError) as e:
        fb.fopd_loss_fwd_bwd_static(*too_many_rows)
    assert e.value.status == 11
    too_many_samples = list(args)
    too_many_samples[12] = fb.FOPD_STATIC_MAX_SAMPLES + 1
    with pytest.raises(fb.FopdError) as e:
        fb.fopd_loss_fwd_bwd_static(*too_many_samples)
    assert e.value.status == 11
    # a token id out of range: the flag comes back through flags_out, and the next call starts clean
    flags = torch.zeros(1, dtype=torch.int32, device=DEV)
    bad = w["token_ids"].clone()
    bad[3] = V
    with_bad = list(args)
    with_bad[5] = bad
    with_bad[-1] = flags
    fb.fopd_loss_fwd_bwd_static(*with_bad)
    torch.cuda.synchronize()
    assert int(flags) == 1 and fb.fopd_flags_status(int(flags)) == 6
    assert float(lp.logp[3]) == 0.0 and not bool(lp.dlogits[3].any())
    args[-1] = flags
    fb.fopd_loss_fwd_bwd_static(*args)
    torch.cuda.synchronize()
    assert int(flags) == 0
