"""GPU parity of fopd_lm_head_loss_fwd_bwd: the second loop of Algorithm 1 on logits that are the projection of
the hidden states and exist only chunk by chunk, with the gradient carried to the hidden states and to the
projection matrix on the matrix cores.  Oracle: lm_head_loss_fwd_bwd (float64)."""

import numpy as np
import pytest
import torch

from harness import workloads as wl
from oracle import fopd_oracle as orc
from paper_2605_17862_amd import binding as fb
from parity_util import assert_close, coef_uncertainty, np64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print("[gpu-projection-loss] " + msg, flush=True)


def _aligned(nbytes):
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=DEV)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + nbytes]
    fb.fopd_workspace_init(ws)
    return ws


def _as_passed(hp):
    """The hyper-parameters as the library receives them: a struct of four floats.  The oracle gets the same
    values (0.05 as a float is 7e-10 above 0.05, which decides the gate when f_i is exactly 1/20)."""
    return tuple(float(np.float32(x)) for x in hp)


def _scores_from_the_oracle(w, hp):
    """First loop of Algorithm 1 in the oracle (float64), rounded to the float32 array both sides receive."""
    hp = _as_passed(hp)
    d = w["d"]
    lse, lp = orc.lm_head_token_logprobs(np64(w["hidden"])[:, :d], np64(w["weight"])[:, :d], np64(w["token_ids"]),
                                         np64(w["mask"]))
    _, _, _, k_roll, k_sup = orc.token_terms(lp, np64(w["behav_logp"]), np64(w["teacher_logp"]), None)
    cu = orc.segment_offsets(w["seq_lens_host"])
    D_roll, D_sup, _, _, _ = orc.sample_statistics(lp, np64(w["teacher_logp"]), k_roll, k_sup, np64(w["mask"]), cu)
    _, _, n_valid = orc.roll_coverage(np64(w["mask"]), cu)
    f = orc.freshness_score(D_roll, D_sup, w["lag_host"], n_valid, hp[0], hp[1])
    return f.astype(np.float32)


def _run(w, hp, g, rows_chunk, f32_scores, accumulate=False, dweight=None, counts=None, pad_h=0, pad_w=0):
    """pad_h / pad_w: extra columns in the rows of dhidden / dweight (they must come back untouched)."""
    T, V, d, B = w["T"], w["V"], w["d"], w["B"]
    ws = _aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk))
    dh_full = torch.full((T, d + pad_h), 7.0, device=DEV)
    dw_full = torch.full((V, d + pad_w), 7.0, device=DEV) if dweight is None else dweight
    out = dict(loss=torch.full((1,), 7.0, device=DEV), weights=torch.empty(B, device=DEV),
               logp=torch.full((T,), 7.0, device=DEV), lse=torch.full((T,), 7.0, device=DEV), ws=ws)
    n_in, nr_in = (None, None) if counts is None else counts
    fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                 w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp,
                                 torch.from_numpy(f32_scores).to(DEV), n_in, nr_in, g, rows_chunk, out["loss"],
                                 out["weights"], out["logp"], out["lse"], dh_full, d + pad_h, dw_full,
                                 dw_full.shape[1], accumulate, ws)
    torch.cuda.synchronize()
    assert fb.fopd_workspace_status(ws) == (0, 0)
    if pad_h:
        assert bool((dh_full[:, d:] == 7.0).all())
    if pad_w and dweight is None:
        assert bool((dw_full[:, d:] == 7.0).all())
    out["dhidden"], out["dweight"] = dh_full[:, :d], dw_full[:, :d]
    return out


def _compare(w, hp, g, out, f32_scores, check_scale=True):
    hp = _as_passed(hp)
    d, V, B = w["d"], w["V"], w["B"]
    H, W = np64(w["hidden"])[:, :d], np64(w["weight"])[:, :d]
    mask = np64(w["mask"])
    ref = orc.lm_head_loss_fwd_bwd(H, W, np64(w["token_ids"]), mask, np64(w["behav_logp"]), np64(w["teacher_logp"]),
                                   w["seq_lens_host"], w["lag_host"], f32_scores.astype(np.float64), hp[2], hp[3], g)
    assert_close("logp", np64(out["logp"]), ref["logp"], atol=1e-4)
    assert_close("lse", np64(out["lse"]), ref["lse"], atol=1e-4)
    assert_close("weights", np64(out["weights"]), ref["weights"], rtol=1e-6, atol=1e-9)
    # each l_i is a mean of fp32 log-probs, good to 1e-6 absolute: so is their weighted mean
    assert abs(float(out["loss"]) - ref["loss"]) <= 1e-5 * abs(ref["loss"]) + 1e-6 * float(np.mean(ref["weights"])) + 1e-12, (
        float(out["loss"]), ref["loss"])
    # The gradient rows the GPU contracts are bf16 values within 2 ulp (plus the coefficient's own uncertainty)
    # of the oracle's bf16 rows; each output is a sum of such rows times exact bf16 operands, in fp32:
    #   |dH - dH_ref| <= sum_v (2^-7 |g| + |p - onehot| eps_c) |W|  +  2^-20 sum_v |g| |W|
    eps_c = coef_uncertainty(ref, hp, g, B, mask)
    pm = np.exp(ref["logits"] - ref["lse"][:, None])
    pm[np.arange(len(pm)), np64(w["token_ids"])] -= 1.0
    pm[mask == 0] = 0.0
    dg = 2.0 ** -7 * np.abs(ref["dlogits"]) + np.abs(pm) * eps_c[:, None] + 2.0 ** -20 * np.abs(ref["dlogits"])
    lim_h = dg @ np.abs(W) + 1e-30
    lim_w = dg.T @ np.abs(H) + 1e-30
    got_h, got_w = np64(out["dhidden"]), np64(out["dweight"])
    err_h, err_w = np.abs(got_h - ref["dhidden"]), np.abs(got_w - ref["dweight"])
    assert np.all(err_h <= lim_h), "dhidden: worst error / bound %.3f at %s" % (
        float((err_h / lim_h).max()), np.unravel_index(np.argmax(err_h / lim_h), err_h.shape))
    assert np.all(err_w <= lim_w), "dweight: worst error / bound %.3f at %s" % (
        float((err_w / lim_w).max()), np.unravel_index(np.argmax(err_w / lim_w), err_w.shape))
    # what is actually observed, against the scale of the result (the bound above is a worst case)
    rel_h = float(err_h.max() / max(np.abs(ref["dhidden"]).max(), 1e-300))
    rel_w = float(err_w.max() / max(np.abs(ref["dweight"]).max(), 1e-300))
    _say("max |err| / max |value|: dhidden %.2e, dweight %.2e; worst err / bound: %.3f, %.3f"
         % (rel_h, rel_w, float((err_h / lim_h).max()), float((err_w / lim_w).max())))
    if check_scale:
        assert rel_h < 2e-3 and rel_w < 2e-3
        assert np.any(got_h[mask != 0])
    assert not np.any(got_h[mask == 0])
    return ref


CASES = {
    # T-split, d, V, ldh, ldw, masked_every, rows_chunk: ragged tiles on every side, several chunks, a ragged last chunk
    "ragged": ((90, 130, 80), 128, 1000, 136, 128, 7, 128),
    "one_chunk": ((40, 60), 64, 5003, 64, 72, 0, 256),
    "exact_tiles": ((256, 256), 192, 2048, 192, 192, 0, 256),
    "wide_vocab": ((150, 170, 200), 256, 40000, 256, 256, 5, 192),
    "full_vocab": ((300, 350, 400), 256, 151936, 256, 256, 9, 512),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_projection_loss_and_gradients(name):
    seq, d, V, ldh, ldw, every, rows_chunk = CASES[name]
    T = sum(seq)
    _say("%s: T=%d d=%d V=%d chunks of %d rows" % (name, T, d, V, rows_chunk))
    h = wl.generate_lm_head(T, d, V, DEV, seed=5, masked_every=every, ldh=ldh, ldw=ldw)
    lag = [0, 3, 40][:len(seq)]                       # the third sample, where there is one, is gated
    w = wl.attach_loss_inputs(h, seq, lag, seed=5)
    hp, g = (1.0, 1.0, 0.05, 0.3), 1.7
    f = _scores_from_the_oracle(w, hp)
    out = _run(w, hp, g, rows_chunk, f)
    ref = _compare(w, hp, g, out, f)
    if len(seq) == 3:
        assert ref["weights"][2] == 0.0 and float(out["weights"][2]) == 0.0
        assert not bool(out["dhidden"][seq[0] + seq[1]:].any())


def test_projection_loss_accumulates_into_dweight_and_ignores_the_chunk_size():
    seq, d, V = (70, 50), 128, 3000
    T = sum(seq)
    h = wl.generate_lm_head(T, d, V, DEV, seed=9, masked_every=6)
    w = wl.attach_loss_inputs(h, seq, [1, 2], seed=9)
    hp, g = (1.0, 1.0, 0.0, 0.2), 1.0
    f = _scores_from_the_oracle(w, hp)
    one = _run(w, hp, g, 1024, f)                                 # a single chunk
    many = _run(w, hp, g, 64, f)                                  # two chunks (64 + 56 rows)
    assert torch.equal(one["logp"], many["logp"]) and torch.equal(one["dhidden"], many["dhidden"])
    assert torch.allclose(one["dweight"], many["dweight"], rtol=1e-5, atol=1e-9)     # fp32 sums over rows, other order
    assert abs(float(one["loss"]) - float(many["loss"])) <= 2e-6 * abs(float(one["loss"]))
    base = torch.full((V, d), 0.5, device=DEV)
    acc = _run(w, hp, g, 64, f, accumulate=True, dweight=base.clone())
    assert torch.allclose(acc["dweight"], many["dweight"] + 0.5, rtol=1e-6, atol=1e-7)
    # counts passed in instead of taken from the mask: the same result
    cu = orc.segment_offsets(w["seq_lens_host"])
    n = torch.from_numpy(orc.trainable_counts(np64(w["mask"]), cu)).to(DEV)
    given = _run(w, hp, g, 64, f, counts=(n, None))
    assert torch.equal(given["dhidden"], many["dhidden"]) and torch.equal(given["dweight"], many["dweight"])


@pytest.mark.parametrize("seq,rows_chunk,lag", [((90, 130, 80), 192, (0, 3, 40)), ((40, 0, 60, 30, 50, 70), 128, (0, 1, 2, 45, 0, 3)),
                                                ((64, 64), 64, (1, 0)), ((50, 0, 0), 64, (0, 0, 0))])
def test_projection_loss_forms_the_scores_itself_when_given_none(seq, rows_chunk, lag):
    """freshness_in = None: chunks gather whole samples and the scores come from the chunk's own log-probs, as in
    fopd_loss_fwd_bwd without scores.  The scores are checked against the oracle's (1e-5 relative), everything
    else against the oracle evaluated at the scores the call reports; and the call with those scores supplied
    gives the same gradients."""
    T, d, V = sum(seq), 128, 3000
    _say("scores formed inside the call: samples %s, chunks of at most %d rows" % (list(seq), rows_chunk))
    h = wl.generate_lm_head(T, d, V, DEV, seed=21, masked_every=6)
    w = wl.attach_loss_inputs(h, seq, list(lag), seed=21)
    hp, g, B = (1.0, 1.0, 0.05, 0.3), 1.3, len(seq)
    ws = _aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk))
    out = dict(loss=torch.full((1,), 7.0, device=DEV), weights=torch.full((B,), 7.0, device=DEV),
               freshness=torch.full((B,), 7.0, device=DEV), logp=torch.full((T,), 7.0, device=DEV),
               lse=torch.full((T,), 7.0, device=DEV), dhidden=torch.full((T, d), 7.0, device=DEV),
               dweight=torch.full((V, d), 7.0, device=DEV))
    fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                 w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, None, None, None, g,
                                 rows_chunk, out["loss"], out["weights"], out["logp"], out["lse"], out["dhidden"], d,
                                 out["dweight"], d, False, ws, seq_lens_host=w["seq_lens_host"], freshness=out["freshness"])
    torch.cuda.synchronize()
    assert fb.fopd_workspace_status(ws) == (0, 0)
    f_exact = _scores_from_the_oracle(w, hp).astype(np.float64)
    f_gpu = np64(out["freshness"])
    assert_close("freshness", f_gpu, f_exact, rtol=1e-5)
    gated = [i for i in range(B) if 0.0 < f_exact[i] < 0.05]
    if any(x >= 40 for x in lag):
        assert gated and all(float(out["weights"][i]) == 0.0 for i in gated)
    _compare(w, hp, g, out, f_gpu.astype(np.float32), check_scale=T > 60)
    again = _run(w, hp, g, 64, f_gpu.astype(np.float32))          # scores supplied, chunks that cut samples
    assert torch.equal(again["logp"], out["logp"])
    assert torch.allclose(again["dhidden"], out["dhidden"], rtol=2e-2, atol=1e-6 * float(out["dhidden"].abs().max()))
    assert torch.allclose(again["dweight"], out["dweight"], rtol=2e-2, atol=1e-5 * float(out["dweight"].abs().max()))
    # a sample longer than a chunk: the call sweeps the rows twice (log-probs of every chunk first, then the scores
    # of all samples, then the pass as if they had been supplied) and gives what the one-chunk-per-sample call gave
    if max(seq) > 64:
        two = dict(loss=torch.full((1,), 7.0, device=DEV), weights=torch.full((B,), 7.0, device=DEV),
                   freshness=torch.full((B,), 7.0, device=DEV), logp=torch.full((T,), 7.0, device=DEV),
                   lse=torch.full((T,), 7.0, device=DEV), dhidden=torch.full((T, d), 7.0, device=DEV),
                   dweight=torch.full((V, d), 7.0, device=DEV))
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                     w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, None, None,
                                     None, g, 64, two["loss"], two["weights"], two["logp"], two["lse"],
                                     two["dhidden"], d, two["dweight"], d, False, ws,
                                     seq_lens_host=w["seq_lens_host"], freshness=two["freshness"])
        torch.cuda.synchronize()
        assert fb.fopd_workspace_status(ws) == (0, 0)
        for key in ("logp", "lse", "freshness", "weights", "dhidden"):
            assert torch.equal(two[key], out[key]), key
        assert abs(float(two["loss"]) - float(out["loss"])) <= 2e-6 * abs(float(out["loss"]))
        assert torch.allclose(two["dweight"], out["dweight"], rtol=1e-4, atol=1e-6 * float(out["dweight"].abs().max()))


def test_projection_loss_rejects_bad_arguments():
    h = wl.generate_lm_head(64, 64, 100, DEV, seed=1)
    w = wl.attach_loss_inputs(h, (64,), [0], seed=1)
    f = np.ones(1, dtype=np.float32)
    with pytest.raises(fb.FopdError) as e:
        _run(w, (1, 1, 0, 0), 1.0, 100, f)                        # rows_chunk not a multiple of 64
    assert e.value.status == 2
    ws = _aligned(1024)
    t = torch.empty(64, device=DEV)
    with pytest.raises(fb.FopdError) as e:
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], 64, w["weight"], 64, 64, 100, 64, w["token_ids"], None, w["behav_logp"],
                                     w["teacher_logp"], w["seq_lens"], w["lag"], 1, (1, 1, 0, 0),
                                     torch.ones(1, device=DEV), None, None, 1.0, 64, t[:1], None, t, t.clone(),
                                     torch.empty(64, 64, device=DEV), 64, torch.empty(100, 64, device=DEV), 64, 0, ws)
    assert e.value.status == 5                                     # workspace too small


@pytest.mark.parametrize("workload", ["reasoning", "tooluse"])
def test_projection_loss_at_benchmark_size_sampled_rows(workload):
    """The benchmark's shape (rows, mask and lags of the reasoning workload, and of the tool-use one, a third of whose
    rows are masked observation spans; d = 4096, V = 151,936, chunks of 8192 rows).  The scores are an input of this call (Algorithm 1 computes them in its first loop), so seeded values
    are supplied; the oracle then gives, row by row, the log-prob, the coefficient, the bf16 gradient row and its
    contraction with the projection matrix for sampled rows.  dweight is tied to dhidden by the identity
    <dhidden, hidden> = sum_{t,v} dz[t,v] z[t,v] = <dweight, weight>, which holds at any size."""
    seq, mask = wl.structure_only(workload, seed=0)
    T, d, V, B, rows_chunk = int(seq.sum()), 4096, 151936, len(seq), 8192
    _say("benchmark size (%s): T=%d (%d masked) d=%d V=%d, %d chunks: generating ..."
         % (workload, T, int((mask == 0).sum()), d, V, (T + rows_chunk - 1) // rows_chunk))
    lag = np.random.RandomState(0).randint(0, 5, size=B).astype(np.int32)
    w = wl.attach_loss_inputs(wl.generate_lm_head(T, d, V, DEV, seed=0), seq, lag, seed=0)
    w["mask"] = torch.from_numpy(mask).to(DEV)
    hp, g = (1.0, 1.0, 0.05, 0.1), 1.0
    f = np.random.RandomState(5).uniform(0.0, 1.0, size=B).astype(np.float32)
    f[3] = 0.01                                                   # one sample gated by the threshold
    _say("running the call")
    out = _run(w, hp, g, rows_chunk, f)
    cu = orc.segment_offsets(seq)
    n = orc.trainable_counts(mask, cu)
    wts = orc.freshness_weights(f.astype(np.float64), hp[2], n)
    assert_close("weights", np64(out["weights"]), wts, rtol=1e-6, atol=1e-9)
    W64 = np64(w["weight"])
    rs = np.random.RandomState(11)
    rows = sorted(set(rs.randint(0, T, size=10).tolist() + [0, T - 1, int(cu[3]) + 1, rows_chunk - 1, rows_chunk]))
    live_rows = np.flatnonzero(mask != 0)
    rows = sorted(set(rows + [int(live_rows[0]), int(live_rows[-1]), int(live_rows[len(live_rows) // 2])]))
    lb, lq, y = np64(w["behav_logp"]), np64(w["teacher_logp"]), np64(w["token_ids"])
    worst = 0.0
    for t in rows:
        if mask[t] == 0:                                          # a masked row: no log-prob, no gradient row
            assert float(out["logp"][t]) == 0.0 and float(out["lse"][t]) == 0.0 and not bool(out["dhidden"][t].any())
            continue
        i = int(np.searchsorted(cu, t, side="right") - 1)
        h = np64(w["hidden"][t])
        z = orc.lm_head_logits(h[None, :], W64)
        lse, lp = orc.token_logprobs(z, y[t:t + 1], None)
        assert abs(float(out["logp"][t]) - lp[0]) <= 1e-4 and abs(float(out["lse"][t]) - lse[0]) <= 1e-4
        delta, rho, adv, _, _ = orc.token_terms(lp, lb[t:t + 1], lq[t:t + 1], None)
        c = g * wts[i] / (B * int(n[i])) * (adv[0] - hp[3] * rho[0] * delta[0])
        grow = orc.round_to_bf16(orc.dlogits_row(z[0], int(y[t]), lse[0], c))
        want = grow @ W64
        pm = np.exp(z[0] - lse[0])
        pm[int(y[t])] -= 1.0
        eps_c = abs(g) / (B * int(n[i])) * wts[i] * 4e-6
        lim = (2.0 ** -7 * np.abs(grow) + np.abs(pm) * eps_c + 2.0 ** -20 * np.abs(grow)) @ np.abs(W64) + 1e-30
        got = np64(out["dhidden"][t])
        err = np.abs(got - want)
        assert np.all(err <= lim), "dhidden row %d: worst error / bound %.3f" % (t, float((err / lim).max()))
        if wts[i] == 0.0:
            assert not np.any(got)
        else:
            worst = max(worst, float(err.max() / np.abs(want).max()))
    _say("%d sampled rows ok; max |err| / max |row| of dhidden %.2e" % (len(rows), worst))
    assert worst < 2e-3
    lhs = float((out["dhidden"].double() * w["hidden"].double()).sum())
    rhs = float((out["dweight"].double() * w["weight"].double()).sum())
    scale = float((out["dhidden"].double() * w["hidden"].double()).abs().sum())
    _say("<dhidden, hidden> = %.9e, <dweight, weight> = %.9e (sum of magnitudes %.3e)" % (lhs, rhs, scale))
    assert abs(lhs - rhs) <= 1e-5 * scale
    # the loss is the sum of the per-row terms of the library's own log-probs
    lp_gpu = np64(out["logp"])
    per_row_w = np.repeat(wts / (B * np.maximum(n, 1)), seq)
    dl = lp_gpu - lb
    terms = per_row_w * ((lp_gpu - lq) + hp[3] * (np.exp(dl) * dl - np.exp(dl) + 1.0))
    L = float(np.sum(terms[mask != 0]))
    assert abs(float(out["loss"]) - L) <= 1e-5 * abs(L)


def test_projection_loss_random_shapes_sweep():
    """Twelve seeded random problems: hidden size, vocabulary, operand and output row pitches (16-byte aligned or
    not), sample count and lengths, masks with one or two aligned sets, lags, chunk size, scale."""
    rs = np.random.RandomState(123)
    for case in range(12):
        d = int(rs.choice([64, 128, 192, 320]))
        V = int(rs.choice([1, 7, 64, 255, 1000, 2049, 4100, 9001]))
        B = int(rs.randint(1, 5))
        seq = [int(x) for x in rs.randint(1, 90, size=B)]
        T = sum(seq)
        ldh, ldw = d + 8 * int(rs.randint(0, 3)), d + 8 * int(rs.randint(0, 3))
        pad_h, pad_w = int(rs.choice([0, 1, 4, 6])), int(rs.choice([0, 3, 4]))
        rows_chunk = int(rs.choice([64, 128, 256]))
        hp = (float(rs.choice([0.0, 1.0])), 1.0, float(rs.choice([0.0, 0.05, 0.3])), float(rs.choice([0.0, 0.2, 1.0])))
        g = float(rs.choice([1.0, -2.0, 0.125]))
        _say("random case %d: T=%d d=%d V=%d ldh=%d ldw=%d out pads %d/%d chunk %d hp=%s g=%g"
             % (case, T, d, V, ldh, ldw, pad_h, pad_w, rows_chunk, hp, g))
        h = wl.generate_lm_head(T, d, V, DEV, seed=200 + case, masked_every=int(rs.choice([0, 3, 5])), ldh=ldh, ldw=ldw)
        if case % 3 == 1:                                   # two different aligned sets among the kept rows
            m = h["mask"].cpu().numpy()
            u = rs.uniform(size=T)
            m = np.where((m != 0) & (u < 0.3), 2, np.where((m != 0) & (u < 0.6), 3, m)).astype(np.uint8)
            h["mask"] = torch.from_numpy(m).to(DEV)
        w = wl.attach_loss_inputs(h, seq, [int(x) for x in rs.randint(0, 25, size=B)], seed=200 + case)
        f = _scores_from_the_oracle(w, hp)
        out = _run(w, hp, g, rows_chunk, f, pad_h=pad_h, pad_w=pad_w)
        _compare(w, hp, g, out, f, check_scale=False)


# ---------------------------------------------------------------------------------------
# the same pass with the teacher stored as k tokens per row
# ---------------------------------------------------------------------------------------

LISTED_CASES = {
    # T-split, d, V, ldh, ldw, masked_every, rows_chunk, k
    "ragged": ((90, 130, 80), 128, 1000, 136, 128, 7, 192, 12),
    "two_samples_per_chunk": ((60, 70, 50, 40), 64, 5003, 64, 72, 0, 128, 5),
    "full_vocab": ((300, 350, 400), 256, 151936, 256, 256, 9, 512, 64),
}


def _listed_run_and_compare(w, seq, d, V, k, rows_chunk, hp, g, floor, lq_tok=None, lqs_tok=None, gated=None):
    """fopd_lm_head_loss_fwd_bwd_topk_teacher against the oracle on one workload (see the test below for the bound)."""
    from test_gpu_topk_teacher import coefficient_uncertainties, grad_row_want_and_limit
    T, B = sum(seq), len(seq)
    ws = _aligned(fb.fopd_lm_head_loss_topk_workspace_bytes(T, V, d, B, rows_chunk, k))
    f32 = dict(dtype=torch.float32, device=DEV)
    out = dict(loss=torch.full((1,), 7.0, **f32), fresh=torch.empty(B, **f32), weights=torch.empty(B, **f32),
               logp=torch.full((T,), 7.0, **f32), lse=torch.full((T,), 7.0, **f32), tl=torch.full((T,), 7.0, **f32),
               dh=torch.full((T, d + 8), 7.0, **f32), dw=torch.full((V, d), 7.0, **f32))
    fb.fopd_lm_head_loss_fwd_bwd_topk_teacher(
        w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"], w["behav_logp"], w["list_ids"],
        w["list_logp"], k, floor, lq_tok, lqs_tok, w["seq_lens"], w["lag"], B, hp, w["seq_lens_host"], g, rows_chunk,
        out["loss"], out["fresh"], out["weights"], out["logp"], out["lse"], out["tl"], out["dh"], d + 8, out["dw"], d,
        False, ws)
    torch.cuda.synchronize()
    assert fb.fopd_workspace_status(ws) == (0, 0)
    assert bool((out["dh"][:, d:] == 7.0).all())
    H, W = np64(w["hidden"])[:, :d], np64(w["weight"])[:, :d]
    mask = np64(w["mask"])
    ids, lq, y = np64(w["list_ids"]), np64(w["list_logp"]), np64(w["token_ids"])
    ref = orc.lm_head_loss_fwd_bwd_topk_teacher(H, W, y, mask, np64(w["behav_logp"]), ids, lq, floor,
                                                None if lq_tok is None else np64(lq_tok),
                                                None if lqs_tok is None else np64(lqs_tok),
                                                w["seq_lens_host"], w["lag_host"], hp[0], hp[1], hp[2], hp[3], g)
    assert_close("logp", np64(out["logp"]), ref["logp"], atol=1e-4)
    assert_close("lse", np64(out["lse"]), ref["lse"], atol=1e-4)
    assert_close("freshness", np64(out["fresh"]), ref["freshness"], rtol=1e-5)
    assert_close("weights", np64(out["weights"]), ref["weights"], atol=1e-5 * ref["freshness"] + 1e-12)
    sample_of_row = np.repeat(np.arange(B), np.asarray(seq))
    lim = np.zeros((T, V))
    got_tl = np64(out["tl"])
    worst_tol = 0.0
    for t in range(T):
        m, i = int(mask[t]), int(sample_of_row[t])
        if m == 0 or m == 2:
            assert got_tl[t] == 0.0
        else:
            ell, G = orc.topk_token_loss_row(ref["logits"][t], ids[t], lq[t], floor)
            listed = np.zeros(V, dtype=bool)
            listed[[int(u) for u in ids[t] if 0 <= int(u) < V]] = True
            g_rest = float(G[~listed][0]) if np.any(~listed) else 0.0
            # (the last term: the projected logits carry the fp32 accumulation of d products, a few 1e-6 on each
            # listed log-prob)
            tol = 2e-5 * abs(ell) + 1e-6 * (abs(g_rest) + 3.0) + 2e-6
            worst_tol = max(worst_tol, tol)
            assert abs(got_tl[t] - ell) <= tol, (t, got_tl[t], ell)
        if m == 0 or (ref["c1"][t] == 0.0 and ref["c2"][t] == 0.0):
            continue
        eps_c1, eps_c2 = coefficient_uncertainties(ref, t, i, m, hp, g, B)
        _, lim_row, _ = grad_row_want_and_limit(ref["logits"][t], int(y[t]), ids[t], lq[t], floor, ref["c1"][t],
                                                ref["c2"][t], eps_c1, eps_c2, ref["lse"][t], "bf16")
        lim[t] = lim_row + 2.0 ** -20 * np.abs(ref["dlogits"][t])
    assert abs(float(out["loss"]) - ref["loss"]) <= (1e-5 * abs(ref["loss"]) + float(np.mean(ref["weights"])) * worst_tol
                                                     + 1e-12), (float(out["loss"]), ref["loss"])
    lim_h = lim @ np.abs(W) + 1e-30
    lim_w = lim.T @ np.abs(H) + 1e-30
    got_h, got_w = np64(out["dh"])[:, :d], np64(out["dw"])
    err_h, err_w = np.abs(got_h - ref["dhidden"]), np.abs(got_w - ref["dweight"])
    rel_h = float(err_h.max() / max(np.abs(ref["dhidden"]).max(), 1e-300))
    rel_w = float(err_w.max() / max(np.abs(ref["dweight"]).max(), 1e-300))
    _say("max |err| / max |value|: dhidden %.2e, dweight %.2e; worst err / bound: %.3f, %.3f"
         % (rel_h, rel_w, float((err_h / lim_h).max()), float((err_w / lim_w).max())))
    assert np.all(err_h <= lim_h), "dhidden: worst error / bound %.3f" % float((err_h / lim_h).max())
    assert np.all(err_w <= lim_w), "dweight: worst error / bound %.3f" % float((err_w / lim_w).max())
    assert not np.any(got_h[mask == 0])
    if gated is not None:
        assert ref["weights"][gated] == 0.0 and float(out["weights"][gated]) == 0.0
        a2 = sum(seq[:gated])
        assert not bool(out["dh"][a2:a2 + seq[gated], :d].any())
    return ref, rel_h, rel_w


@pytest.mark.parametrize("name", sorted(LISTED_CASES))
def test_projection_loss_with_listed_teacher(name):
    """fopd_lm_head_loss_fwd_bwd_topk_teacher against the oracle's lm_head_loss_fwd_bwd_topk_teacher: log-probs,
    token loss, scores, weights, loss, and dhidden / dweight within the bound that follows from the tolerance of the
    gradient rows (each a bf16 value within its limit of the oracle's bf16 row; exact bf16 operands; fp32 sums):
    |dH - dH_ref| <= (lim + 2^-20 |g|) |W|, likewise for dweight with |H|."""
    seq, d, V, ldh, ldw, every, rows_chunk, k = LISTED_CASES[name]
    T, B = sum(seq), len(seq)
    _say("listed teacher, %s: T=%d d=%d V=%d k=%d chunks of at most %d rows" % (name, T, d, V, k, rows_chunk))
    h = wl.generate_lm_head(T, d, V, DEV, seed=9, masked_every=every, ldh=ldh, ldw=ldw)
    lag = [0, 3, 40, 1][:B]                            # the third sample is gated
    w = wl.attach_loss_inputs(h, seq, lag, seed=9, teacher_list=(k, 0.6))
    w["list_ids"][1, 0] = -1                            # an unused slot
    if not bool((w["list_ids"][2] == w["token_ids"][2]).any()):
        w["list_ids"][2, k // 2] = w["token_ids"][2]    # a listed sampled token
    hp, g, floor = _as_passed((1.0, 1.0, 0.05, 0.3)), 1.7, 1e-4
    ref, rel_h, rel_w = _listed_run_and_compare(w, seq, d, V, k, rows_chunk, hp, g, floor, gated=2)
    assert rel_h < 2e-3 and rel_w < 2e-3


def test_projection_loss_with_listed_teacher_and_supplied_scores():
    """The listed-teacher pass with scores formed earlier (Algorithm 1 scores the buffer before its minibatch loop):
    given the scores its own scoring-only form reports, the call with freshness_in, whose chunks cut samples, returns
    the loss, token losses, log-probs and gradients of the call that forms the scores itself (the weights differ
    in the last place: float32 scores against the float64 ones used inside)."""
    seq, d, V, k, rows_chunk = (90, 130, 80, 70), 128, 3000, 9, 192
    T, B = sum(seq), len(seq)
    _say("listed teacher with supplied scores: T=%d, chunks of %d rows" % (T, rows_chunk))
    h = wl.generate_lm_head(T, d, V, DEV, seed=23, masked_every=6)
    w = wl.attach_loss_inputs(h, seq, [0, 3, 40, 1], seed=23, teacher_list=(k, 0.6))
    hp, g = _as_passed((1.0, 1.0, 0.05, 0.3)), 1.3
    f32 = dict(dtype=torch.float32, device=DEV)

    def run(fin, chunk, grads=True):
        ws = _aligned(fb.fopd_lm_head_loss_topk_workspace_bytes(T, V, d, B, chunk, k))
        o = dict(loss=torch.full((1,), 7.0, **f32), fresh=torch.full((B,), 7.0, **f32),
                 weights=torch.full((B,), 7.0, **f32), logp=torch.full((T,), 7.0, **f32),
                 lse=torch.full((T,), 7.0, **f32), tl=torch.full((T,), 7.0, **f32),
                 dh=torch.full((T, d), 7.0, **f32) if grads else None, dw=torch.full((V, d), 7.0, **f32) if grads else None)
        fb.fopd_lm_head_loss_fwd_bwd_topk_teacher(
            w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"], w["behav_logp"],
            w["list_ids"], w["list_logp"], k, 1e-4, None, None, w["seq_lens"], w["lag"], B, hp,
            None if fin is not None else w["seq_lens_host"], g, chunk, o["loss"], o["fresh"], o["weights"], o["logp"],
            o["lse"], o["tl"], o["dh"], d, o["dw"], d, False, ws, freshness_in=fin)
        torch.cuda.synchronize()
        assert fb.fopd_workspace_status(ws) == (0, 0)
        return o

    scores = run(None, rows_chunk, grads=False)                   # the scoring loop
    inside = run(None, rows_chunk)                                # one call that does both
    given = run(scores["fresh"].clone(), 64)                      # the minibatch call, chunks that cut samples
    assert float(given["weights"][2]) == 0.0 and not bool(given["dh"][220:300].any())
    for key in ("logp", "lse", "tl", "fresh"):
        assert torch.equal(given[key], inside[key]), key
    assert torch.allclose(given["weights"], inside["weights"], rtol=1e-6, atol=1e-9)
    assert abs(float(given["loss"]) - float(inside["loss"])) <= 1e-5 * abs(float(inside["loss"]))
    for key in ("dh", "dw"):
        scale = float(inside[key].abs().max())
        assert torch.allclose(given[key], inside[key], rtol=2e-2, atol=1e-5 * scale), key
    # no scores and chunks shorter than the samples: two sweeps inside the call, the same float64 scores
    swept = run(None, 64)
    for key in ("logp", "lse", "tl", "fresh", "weights", "dh"):
        assert torch.equal(swept[key], inside[key]), key
    assert abs(float(swept["loss"]) - float(inside["loss"])) <= 2e-6 * abs(float(inside["loss"]))
    assert torch.allclose(swept["dw"], inside["dw"], rtol=1e-4, atol=1e-6 * float(inside["dw"].abs().max()))


def test_projection_loss_with_listed_teacher_random_sweep():
    """Ten seeded random problems: sample count and lengths, hidden size, vocabulary, list length, rows per chunk,
    masks with two aligned sets, lags, hyper-parameters, upstream scale, with and without the two sampled-token
    teacher arrays that give D^sup."""
    rs = np.random.RandomState(123)
    for case in range(10):
        B = int(rs.randint(1, 5))
        seq = tuple(int(x) for x in rs.randint(1, 90, size=B))
        T = sum(seq)
        d = int(rs.choice([64, 128, 192]))
        V = int(rs.choice([40, 257, 1000, 4099]))
        k = int(min(V, rs.choice([1, 3, 16, 70])))
        rows_chunk = int(rs.choice([64, 128, 256]))
        rows_chunk = max(rows_chunk, (max(seq) + 63) // 64 * 64)
        hp = _as_passed((float(rs.choice([0.0, 0.5, 2.0])), float(rs.choice([0.0, 1.0])),
                         float(rs.choice([0.0, 0.05, 0.2])), float(rs.choice([0.0, 0.1, 1.0]))))
        g = float(rs.choice([1.0, 0.25, -2.0]))
        _say("random case %d: seq=%s d=%d V=%d k=%d chunk=%d hp=%s g=%g" % (case, seq, d, V, k, rows_chunk, hp, g))
        h = wl.generate_lm_head(T, d, V, DEV, seed=300 + case)
        lag = rs.choice([0, 1, 5, 30], size=B).astype(np.int32)
        w = wl.attach_loss_inputs(h, seq, lag, seed=300 + case, teacher_list=(k, 0.6))
        m = rs.choice([0, 1, 1, 1, 2, 3], size=T).astype(np.uint8)
        w["mask"] = torch.from_numpy(m).to(DEV)
        drop = torch.from_numpy(rs.rand(T, k) < 0.1).to(DEV)
        w["list_ids"][drop] = -1
        lq_tok = lqs_tok = None
        if case % 2 == 1:
            lq_tok = w["teacher_logp"]
            lqs_tok = torch.clamp(lq_tok + 0.2 * torch.from_numpy(rs.randn(T).astype(np.float32)).to(DEV), max=0.0)
        _listed_run_and_compare(w, seq, d, V, k, rows_chunk, hp, g, 1e-4, lq_tok, lqs_tok)


def test_projection_scores_only_calls_give_the_full_calls_scores():
    """With dhidden and dweight both NULL the two calls only score the buffer (first loop of Algorithm 1 on projected
    logits): every output they share with the full call is bit-identical to it, and nothing else is written."""
    _say("scores-only calls (no gradient outputs)")
    seq, d, V, k, rows_chunk = (90, 130, 80), 128, 3000, 9, 192
    T, B = sum(seq), len(seq)
    h = wl.generate_lm_head(T, d, V, DEV, seed=12, masked_every=6)
    w = wl.attach_loss_inputs(h, seq, [0, 3, 40], seed=12, teacher_list=(k, 0.6))
    hp, g = _as_passed((1.0, 1.0, 0.05, 0.3)), 1.3
    f32 = dict(dtype=torch.float32, device=DEV)

    def outs():
        return dict(loss=torch.full((1,), 7.0, **f32), fresh=torch.full((B,), 7.0, **f32),
                    weights=torch.full((B,), 7.0, **f32), logp=torch.full((T,), 7.0, **f32),
                    lse=torch.full((T,), 7.0, **f32), tl=torch.full((T,), 7.0, **f32))

    def listed(o, dh, dw):
        ws = _aligned(fb.fopd_lm_head_loss_topk_workspace_bytes(T, V, d, B, rows_chunk, k))
        fb.fopd_lm_head_loss_fwd_bwd_topk_teacher(
            w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"], w["behav_logp"],
            w["list_ids"], w["list_logp"], k, 1e-4, None, None, w["seq_lens"], w["lag"], B, hp, w["seq_lens_host"], g,
            rows_chunk, o["loss"], o["fresh"], o["weights"], o["logp"], o["lse"], o["tl"], dh, d, dw, d, False, ws)
        torch.cuda.synchronize()
        assert fb.fopd_workspace_status(ws) == (0, 0)

    def sampled(o, dh, dw):
        ws = _aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk))
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                     w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, None, None, None,
                                     g, rows_chunk, o["loss"], o["weights"], o["logp"], o["lse"], dh, d, dw, d, False, ws,
                                     seq_lens_host=w["seq_lens_host"], freshness=o["fresh"])
        torch.cuda.synchronize()
        assert fb.fopd_workspace_status(ws) == (0, 0)

    for call, keys in ((listed, ("loss", "fresh", "weights", "logp", "lse", "tl")),
                       (sampled, ("loss", "fresh", "weights", "logp", "lse"))):
        full, only = outs(), outs()
        call(full, torch.empty(T, d, **f32), torch.empty(V, d, **f32))
        call(only, None, None)
        for key in keys:
            assert torch.equal(full[key], only[key]), key
        assert bool((only["fresh"] != 7.0).all()) and bool((only["logp"] != 7.0).all())
    # the weight gradient without the hidden one, or scoring with scores supplied, is refused
    o = outs()
    with pytest.raises(fb.FopdError):
        listed(o, None, torch.empty(V, d, **f32))
    with pytest.raises(fb.FopdError):
        ws = _aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk))
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                     w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, o["fresh"], None,
                                     None, g, rows_chunk, o["loss"], o["weights"], o["logp"], o["lse"], None, d, None, d,
                                     False, ws)


# ---------------------------------------------------------------------------------------
# masked spans (observations, prompts): their rows are left out of the contractions
# ---------------------------------------------------------------------------------------

def _span_mask(T, dead, rs):
    """All ones, then a few 2s and 3s (two aligned sets), then zeros on the given [start, stop) spans."""
    m = rs.choice([1, 1, 1, 2, 3], size=T).astype(np.uint8)
    for a, b in dead:
        m[a:b] = 0
    return m


def test_projection_loss_leaves_masked_spans_out_of_the_contractions():
    """Long masked spans, as the observation turns of a tool-use buffer: a first chunk with no live row at all, a
    chunk in the middle with none, a masked tail, a sample with no live row, and a sample that the freshness weight
    gates out (log-probs but no gradient rows).  The three forms of the pass (scores supplied, scores formed inside,
    listed teacher) against the oracle, then each against itself with the compaction of live rows and of gradient
    rows switched off: the same log-probs, scores, loss and dhidden rows bit for bit (each row's
    contraction does not depend on where the row sits), dweight up to the order of the fp32 sum over rows."""
    seq, d, V, k, rows_chunk = (300, 90, 260, 250), 128, 3000, 9, 128
    T, B = sum(seq), len(seq)
    rs = np.random.RandomState(77)
    dead = [(0, 150), (200, 230), (300, 390), (512, 640), (700, 701), (880, 900)]
    _say("masked spans %s of T=%d rows, samples %s, chunks of %d rows" % (dead, T, list(seq), rows_chunk))
    h = wl.generate_lm_head(T, d, V, DEV, seed=31)
    h["mask"] = torch.from_numpy(_span_mask(T, dead, rs)).to(DEV)
    w = wl.attach_loss_inputs(h, seq, [0, 1, 40, 2], seed=31, teacher_list=(k, 0.6))     # the third sample is gated
    hp, g = _as_passed((1.0, 1.0, 0.05, 0.3)), 1.3
    f32 = dict(dtype=torch.float32, device=DEV)

    def scored(chunk):
        f = _scores_from_the_oracle(w, hp)
        out = _run(w, hp, g, chunk, f, pad_h=4)
        return out, f

    def unscored(chunk):
        ws = _aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, chunk))
        out = dict(loss=torch.full((1,), 7.0, **f32), weights=torch.full((B,), 7.0, **f32),
                   freshness=torch.full((B,), 7.0, **f32), logp=torch.full((T,), 7.0, **f32),
                   lse=torch.full((T,), 7.0, **f32), dhidden=torch.full((T, d), 7.0, **f32),
                   dweight=torch.full((V, d), 7.0, **f32))
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                     w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, None, None, None,
                                     g, chunk, out["loss"], out["weights"], out["logp"], out["lse"], out["dhidden"], d,
                                     out["dweight"], d, False, ws, seq_lens_host=w["seq_lens_host"],
                                     freshness=out["freshness"])
        torch.cuda.synchronize()
        assert fb.fopd_workspace_status(ws) == (0, 0)
        return out

    def listed(chunk):
        ws = _aligned(fb.fopd_lm_head_loss_topk_workspace_bytes(T, V, d, B, chunk, k))
        out = dict(loss=torch.full((1,), 7.0, **f32), freshness=torch.full((B,), 7.0, **f32),
                   weights=torch.full((B,), 7.0, **f32), logp=torch.full((T,), 7.0, **f32),
                   lse=torch.full((T,), 7.0, **f32), tl=torch.full((T,), 7.0, **f32),
                   dhidden=torch.full((T, d), 7.0, **f32), dweight=torch.full((V, d), 7.0, **f32))
        fb.fopd_lm_head_loss_fwd_bwd_topk_teacher(
            w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"], w["behav_logp"],
            w["list_ids"], w["list_logp"], k, 1e-4, None, None, w["seq_lens"], w["lag"], B, hp, w["seq_lens_host"], g,
            chunk, out["loss"], out["freshness"], out["weights"], out["logp"], out["lse"], out["tl"], out["dhidden"], d,
            out["dweight"], d, False, ws)
        torch.cuda.synchronize()
        assert fb.fopd_workspace_status(ws) == (0, 0)
        return out

    # against the oracle
    out_s, f = scored(rows_chunk)
    ref = _compare(w, hp, g, out_s, f)
    assert ref["weights"][1] == 0.0 and float(out_s["weights"][1]) == 0.0          # the sample with no live row
    assert ref["weights"][2] == 0.0 and float(out_s["weights"][2]) == 0.0          # the gated one: log-probs, no gradient
    assert bool(out_s["logp"][400:500].any()) and not bool(out_s["dhidden"][390:650].any())
    dead_rows = torch.from_numpy(np64(w["mask"]) == 0).to(DEV)
    assert not bool(out_s["logp"][dead_rows].any()) and not bool(out_s["lse"][dead_rows].any())
    out_u = unscored(320)
    _compare(w, hp, g, out_u, np64(out_u["freshness"]).astype(np.float32))
    _listed_run_and_compare(w, seq, d, V, k, 320, hp, g, 1e-4)
    out_l = listed(320)
    # against the same calls on all rows
    try:
        fb.fopd_set_option("lm_head_compact", 0)
        all_s, _ = scored(rows_chunk)
        all_u, all_l = unscored(320), listed(320)
    finally:
        fb.fopd_set_option("lm_head_compact", 1)
    for name, got, want in (("scores supplied", out_s, all_s), ("scores formed inside", out_u, all_u),
                            ("listed teacher", out_l, all_l)):
        for key in sorted(set(got) & set(want) - {"ws", "dweight"}):
            assert torch.equal(got[key], want[key]), (name, key)
        scale = float(want["dweight"].abs().max())
        assert torch.allclose(got["dweight"], want["dweight"], rtol=1e-4, atol=1e-6 * scale), name


def test_projection_loss_without_the_weight_gradient():
    """dweight = NULL (a head that is not trained): everything else bit for bit as in the full call."""
    seq, d, V, rows_chunk = (90, 130, 80), 128, 3000, 128
    T, B = sum(seq), len(seq)
    _say("pass through the projection without dL/dweight")
    h = wl.generate_lm_head(T, d, V, DEV, seed=17, masked_every=6)
    w = wl.attach_loss_inputs(h, seq, [0, 3, 40], seed=17)
    hp, g = _as_passed((1.0, 1.0, 0.05, 0.3)), 1.3
    f = _scores_from_the_oracle(w, hp)
    full = _run(w, hp, g, rows_chunk, f)
    ws = _aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk))
    f32 = dict(dtype=torch.float32, device=DEV)
    out = dict(loss=torch.full((1,), 7.0, **f32), weights=torch.empty(B, **f32), logp=torch.full((T,), 7.0, **f32),
               lse=torch.full((T,), 7.0, **f32), dhidden=torch.full((T, d), 7.0, **f32))
    fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                 w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp,
                                 torch.from_numpy(f).to(DEV), None, None, g, rows_chunk, out["loss"], out["weights"],
                                 out["logp"], out["lse"], out["dhidden"], d, None, 0, False, ws)
    torch.cuda.synchronize()
    assert fb.fopd_workspace_status(ws) == (0, 0)
    for key in sorted(out):
        assert torch.equal(out[key], full[key]), key


def test_projection_loss_without_per_row_outputs_leaves_gated_samples_out():
    """Scores supplied and logp = lse = NULL (the caller has them from the scoring call): the samples of weight 0 are
    not projected at all.  Loss, weights and both gradients as in the call that returns the log-probs."""
    seq, d, V, rows_chunk = (150, 90, 200, 60), 128, 3000, 128
    T, B = sum(seq), len(seq)
    rs = np.random.RandomState(3)
    _say("scores supplied, no per-row outputs: gated samples left out")
    h = wl.generate_lm_head(T, d, V, DEV, seed=51)
    h["mask"] = torch.from_numpy(_span_mask(T, [(0, 40), (300, 330)], rs)).to(DEV)
    w = wl.attach_loss_inputs(h, seq, [0, 3, 1, 2], seed=51)
    hp, g = _as_passed((1.0, 1.0, 0.05, 0.3)), 1.3
    f = np.array([0.8, 0.04, 0.5, 0.05], dtype=np.float32)         # the second sample gated, the fourth on the threshold
    full = _run(w, hp, g, rows_chunk, f)
    assert float(full["weights"][1]) == 0.0 and float(full["weights"][3]) == 0.0 and float(full["weights"][2]) > 0.0
    ws = _aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk))
    f32 = dict(dtype=torch.float32, device=DEV)
    out = dict(loss=torch.full((1,), 7.0, **f32), weights=torch.empty(B, **f32), dhidden=torch.full((T, d), 7.0, **f32),
               dweight=torch.full((V, d), 7.0, **f32))

    def call(lp, ls, fin):
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                     w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, fin, None, None, g,
                                     rows_chunk, out["loss"], out["weights"], lp, ls, out["dhidden"], d, out["dweight"], d,
                                     False, ws, seq_lens_host=w["seq_lens_host"])

    call(None, None, torch.from_numpy(f).to(DEV))
    torch.cuda.synchronize()
    assert fb.fopd_workspace_status(ws) == (0, 0)
    assert torch.equal(out["weights"], full["weights"]) and torch.equal(out["dhidden"], full["dhidden"])
    assert not bool(out["dhidden"][150:240].any()) and not bool(out["dhidden"][440:].any())
    assert abs(float(out["loss"]) - float(full["loss"])) <= 2e-6 * abs(float(full["loss"]))
    scale = float(full["dweight"].abs().max())
    assert torch.allclose(out["dweight"], full["dweight"], rtol=1e-4, atol=1e-6 * scale)
    # one of the two without the other, or neither without scores, is refused
    lp = torch.empty(T, **f32)
    for args in ((lp, None, torch.from_numpy(f).to(DEV)), (None, None, None)):
        with pytest.raises(fb.FopdError):
            call(*args)


def test_projection_loss_replays_from_a_hip_graph_with_other_masks():
    """The pass enqueues kernels only and keeps the counts of live rows and of gradient rows on the device, so a
    captured call stays right when the mask behind it changes: three replays, each after the mask tensor was
    overwritten (other masked spans; no row masked; every row masked), against eager calls on the same inputs."""
    seq, d, V, rows_chunk = (150, 90, 200), 64, 2000, 128
    T, B = sum(seq), len(seq)
    rs = np.random.RandomState(5)
    _say("HIP graph replay of the pass through the projection with the mask changed between replays")
    h = wl.generate_lm_head(T, d, V, DEV, seed=41)
    h["mask"] = torch.from_numpy(_span_mask(T, [(0, 130), (300, 340)], rs)).to(DEV)
    w = wl.attach_loss_inputs(h, seq, [0, 40, 2], seed=41)
    hp, g = _as_passed((1.0, 1.0, 0.05, 0.3)), 0.7
    f32 = dict(dtype=torch.float32, device=DEV)
    f_in = torch.tensor([0.9, 0.01, 0.3], **f32)                  # the second sample is gated

    def outs():
        return dict(loss=torch.full((1,), 7.0, **f32), weights=torch.full((B,), 7.0, **f32),
                    freshness=torch.full((B,), 7.0, **f32), logp=torch.full((T,), 7.0, **f32),
                    lse=torch.full((T,), 7.0, **f32), dhidden=torch.full((T, d), 7.0, **f32),
                    dweight=torch.full((V, d), 7.0, **f32),
                    ws=_aligned(max(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk),
                                    fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, 256))))

    def call(o, scores):
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                     w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, scores, None,
                                     None, g, rows_chunk if scores is not None else 256, o["loss"], o["weights"],
                                     o["logp"], o["lse"], o["dhidden"], d, o["dweight"], d, False, o["ws"],
                                     seq_lens_host=None if scores is not None else w["seq_lens_host"],
                                     freshness=o["freshness"])

    e1, e2, g1, g2 = outs(), outs(), outs(), outs()
    call(e1, f_in)                                                # (also sets the kernel attributes before the capture)
    call(e2, None)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        call(g1, f_in)
        call(g2, None)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    masks = [_span_mask(T, [(10, 20), (140, 260), (430, 440)], rs), np.ones(T, dtype=np.uint8),
             np.zeros(T, dtype=np.uint8)]
    for rep, m in enumerate(masks):
        w["mask"].copy_(torch.from_numpy(m).to(DEV))              # the same tensor the graph reads
        for o in (e1, e2, g1, g2):
            o["dhidden"].fill_(float(rep))
            o["loss"].fill_(9.0)
        call(e1, f_in)
        call(e2, None)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in (("scores supplied", g1, e1), ("scores formed inside", g2, e2)):
            for key in sorted(set(got) - {"ws"}):
                assert torch.equal(got[key], want[key]), (rep, name, key)
            assert fb.fopd_workspace_status(got["ws"]) == (0, 0)
        live = int((m != 0).sum())
        assert bool(g1["dhidden"].any()) == (live > 0)
        assert int((g1["logp"] != 0).sum()) <= live and not bool(g1["dhidden"][torch.from_numpy(m == 0).to(DEV)].any())


def test_projection_loss_row_numbering_random_sweep():
    """Sixteen seeded random problems for the numbering of live rows and of gradient rows: masks made of random
    spans (some samples fully masked, some chunks without a live row), random supplied scores around the threshold
    (gated samples), chunk sizes that cut samples, ragged row counts.  The call with scores supplied against the
    same call with the numbering switched off (every row through all three contractions): per-row outputs and dhidden
    bit for bit, dweight up to the order of its fp32 sum, the loss to 2e-6; and the call without per-row outputs
    against both."""
    rs = np.random.RandomState(2024)
    f32 = dict(dtype=torch.float32, device=DEV)
    for case in range(16):
        B = int(rs.randint(1, 6))
        seq = tuple(int(x) for x in rs.randint(1, 200, size=B))
        T, d, V = sum(seq), int(rs.choice([64, 128])), int(rs.choice([300, 1000, 2049]))
        rows_chunk = int(rs.choice([64, 128, 256]))
        m = rs.choice([1, 1, 1, 2, 3], size=T).astype(np.uint8)
        for _ in range(int(rs.randint(0, 6))):                    # masked spans
            a = int(rs.randint(0, T))
            m[a:a + int(rs.randint(1, 150))] = 0
        if case % 5 == 4:
            m[:] = 0 if case % 2 == 0 else 1                      # nothing live / nothing masked
        f = rs.choice([0.0, 0.04, 0.05, 0.3, 0.9], size=B).astype(np.float32)
        hp, g = _as_passed((1.0, 1.0, 0.05, float(rs.choice([0.0, 0.3])))), float(rs.choice([1.0, -0.5]))
        _say("numbering case %d: seq=%s d=%d V=%d chunk=%d, %d of %d rows masked, scores %s"
             % (case, seq, d, V, rows_chunk, int((m == 0).sum()), T, f.tolist()))
        h = wl.generate_lm_head(T, d, V, DEV, seed=400 + case)
        h["mask"] = torch.from_numpy(m).to(DEV)
        w = wl.attach_loss_inputs(h, seq, [int(x) for x in rs.randint(0, 5, size=B)], seed=400 + case)
        on = _run(w, hp, g, rows_chunk, f, pad_h=int(rs.choice([0, 3])))
        try:
            fb.fopd_set_option("lm_head_compact", 0)
            off = _run(w, hp, g, rows_chunk, f)
        finally:
            fb.fopd_set_option("lm_head_compact", 1)
        for key in ("logp", "lse", "weights", "dhidden"):
            assert torch.equal(on[key], off[key]), (case, key)
        scale = max(float(off["dweight"].abs().max()), 1e-30)
        assert torch.allclose(on["dweight"], off["dweight"], rtol=1e-4, atol=1e-6 * scale), case
        assert abs(float(on["loss"]) - float(off["loss"])) <= 2e-6 * abs(float(off["loss"])) + 1e-12, case
        if case % 4 == 0:                                         # added to a running sum (kept as it is if nothing is live)
            base = torch.full((V, d), 0.5, device=DEV)
            acc = _run(w, hp, g, rows_chunk, f, accumulate=True, dweight=base.clone())
            assert torch.allclose(acc["dweight"], off["dweight"] + 0.5, rtol=1e-4, atol=1e-6 * scale + 1e-7), case
        # without per-row outputs
        ws = _aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk))
        lean = dict(loss=torch.full((1,), 7.0, **f32), weights=torch.empty(B, **f32),
                    dhidden=torch.full((T, d), 7.0, **f32), dweight=torch.full((V, d), 7.0, **f32))
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], w["ldh"], w["weight"], w["ldw"], T, V, d, w["token_ids"], w["mask"],
                                     w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp,
                                     torch.from_numpy(f).to(DEV), None, None, g, rows_chunk, lean["loss"], lean["weights"],
                                     None, None, lean["dhidden"], d, lean["dweight"], d, False, ws)
        torch.cuda.synchronize()
        assert fb.fopd_workspace_status(ws) == (0, 0)
        assert torch.equal(lean["weights"], off["weights"]) and torch.equal(lean["dhidden"], off["dhidden"]), case
        assert torch.allclose(lean["dweight"], off["dweight"], rtol=1e-4, atol=1e-6 * scale), case
        assert abs(float(lean["loss"]) - float(off["loss"])) <= 2e-6 * abs(float(off["loss"])) + 1e-12, case
