"""Shared pieces of the GPU parity tests: tensor -> float64 adapters for the oracle and the
tolerances, written out where they are applied.

Tolerances.  The kernels sum the vocabulary in fp32 and keep lp, lse in fp32: lp carries up to 1e-6 of
rounding (|lse| < 32) plus a 2e-7 bias from log2(e) held as a float; everything per token and per sample
after that is fp64.  Hence:
  integers (cu_seqlens, n_train, gather_idx)      bit-exact
  logp, lse                                       1e-4 absolute
  freshness, loss                                 1e-5 relative (the loss, mean_i w_i (l_i + lambda D_i): plus what the
                                                  absolute tolerances of w_i and l_i below leave when a weight is
                                                  barely positive or lp - lq nearly cancels)
  weights                                         1e-5 * f_i absolute (w = f - xi cancels near the gate)
  D_roll, D_sup, ell                              2e-5 relative + 1e-9 absolute
  dlogits                                         2 ulp of the storage type (bf16), 2e-5 relative (f32),
                                                  plus the floor |p_v - [v=y]| * eps_c(t), where eps_c is
                                                  the absolute uncertainty of the row coefficient c_t that
                                                  the tolerances on lp (fp32) and f_i already allow
"""

import numpy as np
import torch

from oracle import fopd_oracle as orc

EPS_A = 4e-6        # absolute error allowed on (A_t - lambda rho_t delta_t), from fp32 log-probs
# Per-row full-vocabulary KL: 2e-5 relative plus this absolute term.  The small quantity E_p[e^-d - 1] is a sum of
# e'_v - e_v with each exponential good to one fp32 ulp (6e-8 relative), so its absolute error is up to
# 2 * 6e-8 * max_v p_v: 1.2e-7 for a row dominated by one token that is not the sampled one (those are the 2 rows in
# 32,768 that exceed 3e-8 at the coding workload's size), about 3e-8 typically.  Per-sample means keep 3e-8.
KL_ROW_ATOL = 1.2e-7
EPS_F = 1e-5        # relative error allowed on f_i


def np64(t):
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().double().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def oracle_full(w, hp, grad_scale=1.0, want_dlogits=True, unit_rows=False):
    """The oracle on a whole (small) workload."""
    alpha, beta, xi, lam = hp
    V = w["V"]
    return orc.fopd_loss_fwd_bwd(np64(w["logits"])[:, :V], np64(w["token_ids"]), np64(w["mask"]),
                                 np64(w["behav_logp"]), np64(w["teacher_logp"]), np64(w["teacher_logp_stale"]),
                                 np64(w["seq_lens"]), np64(w["lag"]), alpha, beta, xi, lam, grad_scale,
                                 out_dtype=w["dtype"], want_dlogits=want_dlogits, ld=w["ld"], unit_rows=unit_rows)


def assert_close(name, got, want, rtol=0.0, atol=0.0):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want)
    lim = rtol * np.abs(want) + atol
    bad = ~((err <= lim) | (got == want))          # a NaN on either side fails
    assert not np.any(bad), "%s: %d of %d outside tolerance, worst err %.3e (limit %.3e) at %s" % (
        name, int(bad.sum()), bad.size, float(err[bad].max()), float(lim[bad][np.argmax(err[bad])]),
        np.argwhere(bad)[0])


def coef_uncertainty(ref, hp, grad_scale, n_samples, mask):
    """eps_c(t): how far the row coefficient may move given the allowed errors of lp and f.  The
    coefficient is g w / B ( [sup] A / n_sup - [roll] lambda rho delta / n_roll ); the lp error enters
    through the larger of the two shares, the f error scales the whole coefficient."""
    _, _, xi, lam = hp
    T = len(ref["coef"])
    cu, n, f, w = ref["cu_seqlens"], ref["n_train"], ref["freshness"], ref["weights"]
    n_roll = ref.get("n_roll", n)
    mask = np.asarray(mask)
    out = np.zeros(T)
    for i in range(len(n)):
        if n[i] == 0 or n_roll[i] == 0:
            continue
        a, b = int(cu[i]), int(cu[i + 1])
        sup = ((mask[a:b] != 0) & (mask[a:b] != 2)).astype(np.float64)
        roll = ((mask[a:b] != 0) & (mask[a:b] != 3)).astype(np.float64)
        share = np.maximum(sup / int(n[i]), roll / int(n_roll[i]))
        aeff = np.abs(sup * ref["adv"][a:b] / int(n[i]) - roll * lam * ref["rho"][a:b] * ref["delta"][a:b] / int(n_roll[i]))
        out[a:b] = abs(grad_scale) / n_samples * (w[i] * EPS_A * share + EPS_F * f[i] * aeff)
    return out


# How often the plain bound (2 ulp of the storage type) is not enough and the floor is what lets an element
# pass.  Filled by check_grad_rows; read (and reset) by floor_report().
FLOOR_STATS = dict(elements=0, rows=0, beyond_plain=0, rows_beyond_plain=0, tiny=0, sampled_entry=0,
                   min_rel_uncertainty=np.inf, worst_excess_ulp=0.0)


def _count_floor_use(got, want, err, plain_lim, y, c, eps, half_plain_rel):
    st = FLOOR_STATS
    st["elements"] += got.size
    st["rows"] += 1
    beyond = ~((err <= plain_lim) | (got == want))
    if not np.any(beyond):
        return
    n = int(beyond.sum())
    st["beyond_plain"] += n
    st["rows_beyond_plain"] += 1
    tiny = beyond & (np.abs(want) < 2.0 ** -120)          # bf16/fp32 subnormal range: flushed to zero
    st["tiny"] += int(tiny.sum())
    if beyond[y]:
        st["sampled_entry"] += 1
    rest = beyond & ~tiny
    rest[y] = False
    if np.any(rest):
        # the floor exists because c_t is a difference of O(1) quantities: it may only be needed where the
        # allowed absolute error of c_t is a visible fraction of c_t itself
        rel = eps / max(abs(c), 1e-300)
        assert rel >= half_plain_rel, ("an element needs the floor although its row's coefficient is uncertain by only "
                                       "%.2e relative (c = %.3e)" % (rel, c))
        st["min_rel_uncertainty"] = min(st["min_rel_uncertainty"], rel)
        st["worst_excess_ulp"] = max(st["worst_excess_ulp"], float(np.max(err[rest] / (plain_lim[rest] / 2.0))))


def floor_report(reset=True):
    """(copy of the counters, one-line summary)."""
    st = dict(FLOOR_STATS)
    frac = st["beyond_plain"] / max(st["elements"], 1)
    line = ("dlogits: %d elements in %d rows compared; %d (%.2e of them, in %d rows) are outside the plain 2-ulp bound "
            "and pass through the floor: %d in the subnormal range, %d sampled-token entries, the rest in rows whose "
            "coefficient is uncertain by >= %.1e relative (worst %.1f ulp)"
            % (st["elements"], st["rows"], st["beyond_plain"], frac, st["rows_beyond_plain"], st["tiny"],
               st["sampled_entry"], st["min_rel_uncertainty"], st["worst_excess_ulp"]))
    if reset:
        FLOOR_STATS.update(elements=0, rows=0, beyond_plain=0, rows_beyond_plain=0, tiny=0, sampled_entry=0,
                           min_rel_uncertainty=np.inf, worst_excess_ulp=0.0)
    return st, line


def check_grad_rows(got_rows, z_rows, y, lse, coef, eps_c, store, rows_label=""):
    """got_rows: [R, V] float64 values read back from the GPU; the rest are oracle arrays for the
    same R rows.  Rows whose oracle coefficient is exactly 0 (masked or gated) must be all-zero
    unless eps_c allows a weight that is barely positive."""
    R, V = got_rows.shape
    for r in range(R):
        exact = orc.dlogits_row(z_rows[r], int(y[r]), lse[r], coef[r])
        if coef[r] == 0.0 and eps_c[r] == 0.0:
            assert not np.any(got_rows[r]), "row %s%d must be exactly zero" % (rows_label, r)
            continue
        pm = np.exp(z_rows[r] - lse[r])
        pm[int(y[r])] -= 1.0
        floor = np.abs(pm) * eps_c[r] + 2.0 ** -126
        # the float64 oracle forms p_y - 1 by subtraction: its own rounding (lse carries an error of
        # one float64 ulp of |lse|) is visible when p_y is within 1e-13 of 1
        u = 4.0 * np.spacing(max(abs(lse[r]), 1.0))
        floor[int(y[r])] += (abs(coef[r]) + eps_c[r]) * u
        if store == "bf16":
            want = orc.round_to_bf16(exact)
            lim = 2.0 * orc.bf16_ulp(want) + floor
        else:
            want = orc.round_to_f32(exact)
            lim = 2e-5 * np.abs(want) + floor
        err = np.abs(got_rows[r] - want)
        bad = ~((err <= lim) | (got_rows[r] == want))   # a NaN on either side fails
        assert not np.any(bad), "dlogits row %s%d: %d elements off, worst %.3e vs limit %.3e at v=%d (c=%.3e)" % (
            rows_label, r, int(bad.sum()), float(err[bad].max()), float(lim[np.argmax(err * bad)]),
            int(np.argmax(err * bad)), coef[r])
        _count_floor_use(got_rows[r], want, err, lim - floor, int(y[r]), coef[r], eps_c[r],
                         2.0 ** -8 if store == "bf16" else 1e-5)


def check_grad_rows_full_kl(got_rows, z_rows, zs_rows, y, ref, rows, hp, grad_scale, n_samples, sample_of_row, store,
                            c2_scales_with_weight=False):
    """Gradient rows of the full-vocabulary-KL variant against the oracle.  Tolerance: 2 ulp of the
    storage type plus what the allowed errors of lp (fp32), f_i (1e-5 relative) and of the per-row
    KL / lse difference (4e-6 absolute, fp32 sums) can move the row by."""
    lam = hp[3]
    for k, t in enumerate(rows):
        c1, c2 = ref["c1"][t], ref["c2"][t]
        exact = orc.dlogits_row_full_kl(z_rows[k], zs_rows[k], int(y[k]), ref["lse"][t], ref["lse_stale"][t],
                                        ref["roll_kl"][t], c1, c2)
        i = sample_of_row[t]
        # the smaller of the two aligned-set counts: an upper bound on either share, 0 for an invalid sample
        n = int(min(ref["n_train"][i], ref.get("n_roll", ref["n_train"])[i]))
        f, w = ref["freshness"][i], ref["weights"][i]
        if c1 == 0.0 and c2 == 0.0 and (n == 0 or f < hp[2] * (1 - 1e-4) or ref["lse"][t] == 0.0):
            assert not np.any(got_rows[k]), "row %d must be exactly zero" % t
            continue
        pref = abs(grad_scale) / (n_samples * max(n, 1))
        p = np.exp(z_rows[k] - ref["lse"][t])
        pm = p.copy()
        pm[int(y[k])] -= 1.0
        ld = (z_rows[k] - ref["lse"][t]) - (zs_rows[k] - ref["lse_stale"][t]) - ref["roll_kl"][t]
        eps_c1 = pref * (w * EPS_A + EPS_F * f * abs(ref["adv"][t]))
        eps_c2 = pref * (1.0 if c2_scales_with_weight else lam) * EPS_F * f
        floor = np.abs(pm) * eps_c1 + p * (np.abs(ld) * eps_c2 + abs(c2) * 8e-6) + 2.0 ** -126
        u = 4.0 * np.spacing(max(abs(ref["lse"][t]), 1.0))
        floor[int(y[k])] += (abs(c1) + eps_c1) * u
        if store == "bf16":
            want = orc.round_to_bf16(exact)
            lim = 2.0 * orc.bf16_ulp(want) + floor
        else:
            want = orc.round_to_f32(exact)
            lim = 2e-5 * np.abs(want) + floor
        err = np.abs(got_rows[k] - want)
        bad = ~((err <= lim) | (got_rows[k] == want))   # a NaN on either side fails
        assert not np.any(bad), "full-KL dlogits row %d: %d elements off, worst %.3e vs limit %.3e at v=%d" % (
            t, int(bad.sum()), float(err[bad].max()), float(lim[np.argmax(err * bad)]), int(np.argmax(err * bad)))
