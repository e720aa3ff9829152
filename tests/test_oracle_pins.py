"""Pins for the float64 oracle: closed forms, library routines, brute-force enumeration and
finite differences.  None of these tests touches the GPU or the HIP library.

Each test is chosen so that a plausible slip in the oracle (dropped term, wrong sign or
index, transposed operand, wrong normaliser) makes it fail.
"""

import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import fopd_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------------------------------
# integers
# ---------------------------------------------------------------------------------------

def test_segment_offsets_and_counts_against_python_ints():
    rng = _rng(1)
    seq = rng.integers(0, 9, size=11)
    seq[3] = 0                                   # an empty sample
    cu = orc.segment_offsets(seq)
    assert cu.dtype == np.int64 and cu[0] == 0
    assert list(cu) == [sum(int(s) for s in seq[:i]) for i in range(12)]
    T = int(cu[-1])
    mask = rng.integers(0, 2, size=T).astype(np.uint8)
    n = orc.trainable_counts(mask, cu)
    assert n.dtype == np.int32
    for i in range(11):
        assert int(n[i]) == int(mask[cu[i]:cu[i + 1]].sum())
    assert int(n[3]) == 0


def test_coverage_is_aligned_positions_over_length():
    """m_i = |U_i| / H_i (Algorithm 1, alignment ratios): 3 of 4 rows, 1 of 2 rows, an empty sample."""
    seq = np.array([4, 2, 0], dtype=np.int32)
    mask = np.array([1, 0, 1, 1, 0, 1], dtype=np.uint8)
    z = np.zeros((6, 3))
    y = np.zeros(6, dtype=np.int32)
    lp = np.full(6, -math.log(3.0))
    res = orc.fopd_loss_fwd_bwd(z, y, mask, lp, lp - 0.1, None, seq, np.zeros(3, dtype=np.int32), 1.0, 1.0, 0.0, 0.0)
    np.testing.assert_allclose(res["cover"], [0.75, 0.5, 0.0], rtol=1e-15)
    np.testing.assert_allclose(res["agg"], [2.0 / 3.0, 1.25 / 3.0, 1.25 / 3.0], rtol=1e-15)   # means over all 3 samples
    assert list(res["n_train"]) == [3, 1, 0]


def test_gather_index_is_64_bit_row_major():
    ids = np.array([5, 0, 151935], dtype=np.int32)
    out = orc.gather_index(ids, 151936)
    assert out.dtype == np.int64
    assert list(out) == [5, 151936, 2 * 151936 + 151935]
    # beyond 2^32: row 40000 of a 151936-wide matrix
    big = orc.gather_index(np.arange(40001, dtype=np.int32) % 7, 151936)
    assert int(big[40000]) == 40000 * 151936 + 40000 % 7 > 2 ** 32


# ---------------------------------------------------------------------------------------
# log-softmax
# ---------------------------------------------------------------------------------------

def test_logprobs_match_library_log_softmax():
    rng = _rng(2)
    T, V = 9, 257
    z = rng.normal(0, 3, size=(T, V))
    z[4] *= 200.0                                # large magnitudes: must not overflow
    y = rng.integers(0, V, size=T)
    lse, lp = orc.token_logprobs(z, y, None)
    ref = scipy.special.log_softmax(z, axis=1)
    np.testing.assert_allclose(lp, ref[np.arange(T), y], rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, scipy.special.logsumexp(z, axis=1), rtol=1e-14)
    tref = torch.log_softmax(torch.from_numpy(z), dim=1).numpy()
    np.testing.assert_allclose(lp, tref[np.arange(T), y], rtol=0, atol=1e-12)


def test_logprobs_closed_forms():
    # constant row: lp = -log V whatever the constant
    V = 1000
    z = np.full((2, V), 7.25)
    z[1] = -3e4
    _, lp = orc.token_logprobs(z, np.array([3, 999]), None)
    # lse = const + log V is rounded at the magnitude of the constant (ulp(3e4) = 3.6e-12)
    np.testing.assert_allclose(lp, [-math.log(V)] * 2, rtol=0, atol=1e-11)
    # z = log(1,2,3,4): probabilities 0.1 .. 0.4
    z = np.log(np.array([[1.0, 2.0, 3.0, 4.0]] * 4))
    _, lp = orc.token_logprobs(z, np.array([0, 1, 2, 3]), None)
    np.testing.assert_allclose(np.exp(lp), [0.1, 0.2, 0.3, 0.4], rtol=1e-14)
    # two classes, z = (0, log 3): p = (1/4, 3/4)
    z = np.array([[0.0, math.log(3.0)]] * 2)
    lse, lp = orc.token_logprobs(z, np.array([0, 1]), None)
    np.testing.assert_allclose(lp, [math.log(0.25), math.log(0.75)], rtol=1e-14)
    np.testing.assert_allclose(lse, [math.log(4.0)] * 2, rtol=1e-14)


def test_softmax_rows_sum_to_one_and_masked_rows_are_zero():
    rng = _rng(3)
    z = rng.normal(0, 2, size=(6, 300))
    y = rng.integers(0, 300, size=6)
    mask = np.array([1, 0, 1, 1, 0, 1], dtype=np.uint8)
    lse, lp = orc.token_logprobs(z, y, mask)
    for t in range(6):
        if mask[t]:
            assert abs(np.exp(z[t] - lse[t]).sum() - 1.0) < 1e-13
        else:
            assert lse[t] == 0.0 and lp[t] == 0.0


def test_entropy_closed_forms_and_library():
    import scipy.stats
    V = 512
    z = np.zeros((4, V))
    z[1] = 3.7                                   # uniform rows: H = log V
    z[2, 5] = 800.0                              # one-hot: H = 0
    z[3, :2] = [math.log(3.0), 0.0]
    z[3, 2:] = -np.inf                           # two live classes (3/4, 1/4), the rest excluded
    H = orc.token_entropy(z, np.array([1, 1, 1, 1]))
    np.testing.assert_allclose(H[:2], [math.log(V)] * 2, rtol=1e-13)
    assert abs(H[2]) < 1e-300 + 1e-12
    np.testing.assert_allclose(H[3], -(0.75 * math.log(0.75) + 0.25 * math.log(0.25)), rtol=1e-13)
    rng = _rng(30)
    z = rng.normal(0, 3, size=(5, 300))
    mask = np.array([1, 1, 0, 1, 1], dtype=np.uint8)
    H = orc.token_entropy(z, mask)
    ref = scipy.stats.entropy(scipy.special.softmax(z, axis=1), axis=1)
    np.testing.assert_allclose(H[mask == 1], ref[mask == 1], rtol=1e-12)
    assert H[2] == 0.0 and np.all(H[mask == 1] > 0) and np.all(H <= math.log(300))


def test_token_out_of_range_raises():
    z = np.zeros((1, 4))
    with pytest.raises(ValueError):
        orc.token_logprobs(z, np.array([4]), None)
    with pytest.raises(ValueError):
        orc.token_logprobs(z, np.array([-1]), None)


# ---------------------------------------------------------------------------------------
# estimator k, ratio, advantage
# ---------------------------------------------------------------------------------------

def test_kl_estimator_expectation_equals_enumerated_kl():
    """sum_y pi_r(y) k(log pi_t(y) - log pi_r(y)) = KL(pi_t || pi_r) by enumeration."""
    rng = _rng(4)
    for V in (2, 5, 16):
        zt, zr = rng.normal(0, 1.5, size=V), rng.normal(0, 1.5, size=V)
        pt = np.exp(zt - scipy.special.logsumexp(zt))
        pr = np.exp(zr - scipy.special.logsumexp(zr))
        kl = sum(pt[v] * math.log(pt[v] / pr[v]) for v in range(V))
        kl_rev = sum(pr[v] * math.log(pr[v] / pt[v]) for v in range(V))
        est = 0.0
        for y in range(V):
            d, rho, _, k_roll, _ = orc.token_terms(np.array([math.log(pt[y])]),
                                                   np.array([math.log(pr[y])]),
                                                   np.array([0.0]))
            assert abs(rho[0] - pt[y] / pr[y]) < 1e-12
            assert k_roll[0] >= 0.0
            est += pr[y] * k_roll[0]
        assert abs(est - kl) < 1e-12
        assert abs(est - kl_rev) > 1e-3          # the direction matters: it is not KL(pi_r||pi_t)


def test_k_is_zero_iff_fresh_and_derivative_is_rho_delta():
    lp = np.array([-1.3, -0.2, -7.0])
    d, rho, adv, k_roll, k_sup = orc.token_terms(lp, lp.copy(), lp - 0.5, None)
    assert np.all(d == 0) and np.all(rho == 1.0) and np.all(k_roll == 0.0) and np.all(k_sup == 0.0)
    np.testing.assert_allclose(adv, [-0.5] * 3)
    # dk/d(delta) = rho * delta by central differences
    for delta in (-0.7, -0.01, 0.3, 1.1):
        h = 1e-6
        fd = (orc.kl_estimator(delta + h) - orc.kl_estimator(delta - h)) / (2 * h)
        assert abs(fd - math.exp(delta) * delta) < 1e-8
    # k_sup uses current minus stale teacher log-prob
    lq, lqs = np.array([-0.4]), np.array([-0.9])
    *_, ks = orc.token_terms(np.array([-1.0]), np.array([-1.0]), lq, lqs)
    e = 0.5
    assert abs(ks[0] - (math.exp(e) * e - math.exp(e) + 1)) < 1e-15


def test_on_policy_expected_gradient_is_gradient_of_reverse_kl():
    """sum_y p_y * A_y * (p - e_y) = grad_z KL(softmax(z) || q) = p * (log p - log q - KL)."""
    rng = _rng(5)
    V = 7
    z = rng.normal(0, 1.2, size=V)
    zq = rng.normal(0, 1.2, size=V)
    logp = z - scipy.special.logsumexp(z)
    logq = zq - scipy.special.logsumexp(zq)
    p = np.exp(logp)
    kl = float(np.sum(p * (logp - logq)))
    want = p * (logp - logq - kl)
    got = np.zeros(V)
    lse = scipy.special.logsumexp(z)
    for y in range(V):
        _, _, adv, _, _ = orc.token_terms(np.array([logp[y]]), np.array([logp[y]]), np.array([logq[y]]))
        got += p[y] * orc.dlogits_row(z, y, lse, adv[0])
    np.testing.assert_allclose(got, want, atol=1e-14)


# ---------------------------------------------------------------------------------------
# freshness score, weights, loss
# ---------------------------------------------------------------------------------------

def test_freshness_closed_form_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "freshness_closed_form.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 6
    for tau, dr, ds, a, b, want in rows:
        f = orc.freshness_score([float(dr)], [float(ds)], [int(tau)], [5], float(a), float(b))
        assert abs(f[0] - float(want)) <= 1e-15 * max(1.0, float(want)) + 2e-16


def test_freshness_lag_only_monotone_and_invalid():
    lag = np.arange(0, 12)
    f = orc.freshness_score(np.full(12, 0.3), np.full(12, 0.7), lag, np.full(12, 4), 0.0, 0.0)
    np.testing.assert_allclose(f, 1.0 / (lag + 1.0), rtol=1e-15)       # lag-only special case
    f = orc.freshness_score(np.full(12, 0.3), np.full(12, 0.1), lag, np.full(12, 4), 1.0, 2.0)
    assert np.all(np.diff(f) < 0) and np.all(f > 0) and np.all(f <= 1)
    D = np.linspace(0, 2, 9)
    f_r = orc.freshness_score(D, np.zeros(9), np.zeros(9, int), np.ones(9, int), 1.5, 0.5)
    f_s = orc.freshness_score(np.zeros(9), D, np.zeros(9, int), np.ones(9, int), 1.5, 0.5)
    assert np.all(np.diff(f_r) < 0) and np.all(np.diff(f_s) < 0)
    assert f_r[0] == 1.0 and f_s[0] == 1.0
    np.testing.assert_allclose(f_r, np.exp(-1.5 * np.sqrt(D)), rtol=1e-15)
    np.testing.assert_allclose(f_s, np.exp(-0.5 * np.sqrt(D)), rtol=1e-15)   # alpha/beta not swapped
    f = orc.freshness_score([0.0, 0.0], [0.0, 0.0], [0, 0], [0, 3], 1.0, 1.0)
    assert f[0] == 0.0 and f[1] == 1.0                                  # n_i = 0 -> f_i = 0
    with pytest.raises(ValueError):
        orc.freshness_score([0.0], [0.0], [0], [1], -1.0, 0.0)
    with pytest.raises(ValueError):
        orc.freshness_score([0.0], [0.0], [-1], [1], 1.0, 0.0)


def test_weights_are_relu_of_f_minus_xi():
    f = np.array([0.9, 0.05, 0.049, 0.0, 0.5])
    n = np.array([3, 3, 3, 0, 0])
    w = orc.freshness_weights(f, 0.05, n)
    np.testing.assert_allclose(w, [0.85, 0.0, 0.0, 0.0, 0.0], atol=1e-16)
    w = orc.freshness_weights(f, -0.1, n)       # a negative threshold must not revive invalid samples
    assert w[3] == 0.0 and w[4] == 0.0 and abs(w[1] - 0.15) < 1e-15


def test_loss_normaliser_linearity_and_permutation():
    rng = _rng(6)
    B = 9
    w = rng.uniform(0, 1, B); w[2] = 0.0
    ell = rng.normal(0.2, 0.1, B)
    D = rng.uniform(0, 0.1, B)
    L0 = orc.anchored_loss(w, ell, D, 0.0)
    L1 = orc.anchored_loss(w, ell, D, 1.0)
    L3 = orc.anchored_loss(w, ell, D, 3.0)
    assert abs(L0 - float(np.sum(w * ell)) / B) < 1e-15       # divides by all B, gated included
    assert abs((L3 - L0) - 3.0 * (L1 - L0)) < 1e-15           # linear in lambda
    assert abs((L1 - L0) - float(np.sum(w * D)) / B) < 1e-15
    perm = rng.permutation(B)
    assert orc.anchored_loss(w[perm], ell[perm], D[perm], 0.7) == orc.anchored_loss(w, ell, D, 0.7)


def _hand_worked_two_set_inputs():
    """The inputs of tests/golden/hand_worked_two_sets.txt: integer softmax weights per row, the two aligned
    sets told apart by the mask byte, log-ratios that are +-ln2 / +-ln3 on the rows a set uses and decoys
    (large, different values) on the rows it must not use."""
    ln2, ln3 = math.log(2.0), math.log(3.0)
    weights = [(1, 1, 1, 1), (1, 3, 2, 2), (2, 1, 1, 4), (1, 2, 4, 1), (4, 2, 1, 1), (1, 1, 1, 1), (1, 1, 2, 4),
               (1, 1, 1, 1), (1, 1, 1, 1)]
    z = np.log(np.array(weights, dtype=np.float64))
    y = np.array([0, 1, 3, 2, 0, 2, 2, 1, 1], dtype=np.int32)
    mask = np.array([1, 2, 2, 3, 3, 0, 1, 3, 3], dtype=np.uint8)
    lp = np.array([-2 * ln2, ln3 - 3 * ln2, -ln2, -ln2, -ln2, -2 * ln2, -2 * ln2, -2 * ln2, -2 * ln2])
    delta = np.array([ln2, -ln2, ln3, 2.5, 4.0, 0.3, -ln3, 0.0, 0.0])        # rows 3, 4, 5: decoys
    lp_minus_lq = np.array([ln3, 0.9, -1.1, -ln2, ln2, 0.2, ln3, ln2, ln2])  # rows 1, 2, 5: decoys
    lq_minus_lqs = np.array([ln2, 1.0, -0.25, ln3, -ln2, 2.0, ln2, 0.1, 0.2])  # rows 1, 2, 5: decoys
    lq = lp - lp_minus_lq
    return dict(z=z, y=y, mask=mask, lb=lp - delta, lq=lq, lqs=lq - lq_minus_lqs, lp=lp,
                seq=np.array([4, 3, 2], dtype=np.int32), lag=np.array([1, 0, 0], dtype=np.int32),
                hp=dict(alpha=0.5, beta=0.25, xi=-0.5, lam=0.5), g=2.0, weights=np.array(weights, dtype=np.float64))


def test_hand_worked_case_with_two_different_aligned_sets():
    """Literal values worked by hand from Eq. "kl-diagnostics" (both lines), Eq. "sample-aggregated-loss", Eq.
    "freshness", the aggregates and weights of Sec. 4.2 and Algorithm 1's invalid-sample branch, on a case
    where |U^sup|, |U^roll| and H_i all differ and one sample has U^roll empty while xi < 0.  Nothing here
    re-evaluates a formula: the expected numbers are read from the fixture."""
    want = {}
    for line in open(os.path.join(GOLDEN, "hand_worked_two_sets.txt")):
        if line.strip() and not line.startswith("#"):
            name, *vals = line.split()
            want[name] = np.array([float(v) for v in vals])
    c = _hand_worked_two_set_inputs()
    res = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"], c["lag"],
                                grad_scale=c["g"], **c["hp"])
    np.testing.assert_allclose(res["logp"][c["mask"] != 0], c["lp"][c["mask"] != 0], rtol=0, atol=1e-15)
    assert list(res["n_train"]) == list(want["n_sup"]) and list(res["n_roll"]) == list(want["n_roll"])
    for key in ("D_roll", "D_sup", "ell", "cover", "cover_roll", "freshness", "weights", "agg", "coef"):
        np.testing.assert_allclose(res[key], want[key], rtol=0, atol=2e-16 + 1e-15, err_msg=key)
    assert abs(res["loss"] - want["loss"][0]) <= 1e-15
    assert want["agg"][1] != want["agg"][2]                       # the two coverage means differ in this case
    assert res["weights"][2] == 0.0 and res["freshness"][2] == 0.0 and 0.0 - c["hp"]["xi"] > 0.0
    # one gradient row spelled out: c_2 * (softmax - onehot) with softmax = weights / 8
    np.testing.assert_allclose(res["dlogits_exact"][2], want["coef"][2] * np.array([0.25, 0.125, 0.125, -0.5]),
                               rtol=0, atol=1e-15)
    assert np.all(res["dlogits_exact"][[5, 7, 8]] == 0.0)


# ---------------------------------------------------------------------------------------
# whole pass: tiny brute-force cases
# ---------------------------------------------------------------------------------------

def _tiny_case(seed, V=11, seq=(3, 0, 5, 4), stale=True, lag=(0, 2, 1, 3)):
    rng = _rng(seed)
    seq = np.array(seq, dtype=np.int32)
    T = int(seq.sum())
    z = rng.normal(0, 2, size=(T, V))
    y = rng.integers(0, V, size=T).astype(np.int32)
    mask = (rng.uniform(size=T) < 0.75).astype(np.uint8)
    lp_true = scipy.special.log_softmax(z, axis=1)[np.arange(T), y]
    lb = np.minimum(lp_true + rng.normal(0, 0.2, T), 0.0)
    lq = np.minimum(lp_true + rng.normal(-0.3, 0.5, T), 0.0)
    lqs = np.minimum(lq + rng.normal(0, 0.2, T), 0.0) if stale else None
    return dict(z=z, y=y, mask=mask, lb=lb, lq=lq, lqs=lqs, seq=seq,
                lag=np.array(lag, dtype=np.int32))


def _scalar_reimplementation(c, alpha, beta, xi, lam, g):
    """The same pass with nothing but Python floats and loops (no numpy arithmetic)."""
    z, y, mask = c["z"], c["y"], c["mask"]
    T, V = z.shape
    B = len(c["seq"])
    out_f, out_w, out_D, out_ell = [], [], [], []
    grads = [[0.0] * V for _ in range(T)]
    loss = 0.0
    start = 0
    for i in range(B):
        H = int(c["seq"][i])
        rows = [t for t in range(start, start + H) if mask[t]]
        start += H
        if not rows:
            out_f.append(0.0); out_w.append(0.0); out_D.append(0.0); out_ell.append(0.0)
            continue
        lps = {}
        for t in rows:
            mx = max(float(v) for v in z[t])
            lse = mx + math.log(sum(math.exp(float(v) - mx) for v in z[t]))
            lps[t] = (float(z[t][y[t]]) - lse, lse)
        n = len(rows)
        Dr = sum(math.exp(lps[t][0] - c["lb"][t]) * (lps[t][0] - c["lb"][t])
                 - math.exp(lps[t][0] - c["lb"][t]) + 1.0 for t in rows) / n
        Ds = 0.0
        if c["lqs"] is not None:
            Ds = sum(math.exp(c["lq"][t] - c["lqs"][t]) * (c["lq"][t] - c["lqs"][t])
                     - math.exp(c["lq"][t] - c["lqs"][t]) + 1.0 for t in rows) / n
        el = sum(lps[t][0] - c["lq"][t] for t in rows) / n
        f = math.exp(-alpha * math.sqrt(Dr) - beta * math.sqrt(Ds)) / (int(c["lag"][i]) + 1)
        w = max(f - xi, 0.0)
        loss += w * (el + lam * Dr) / B
        for t in rows:
            lp, lse = lps[t]
            d = lp - c["lb"][t]
            ct = g * w / (B * n) * ((c["lq"][t] - lp) - lam * math.exp(d) * d)
            for v in range(V):
                grads[t][v] = ct * (math.exp(float(z[t][v]) - lse) - (1.0 if v == y[t] else 0.0))
        out_f.append(f); out_w.append(w); out_D.append(Dr); out_ell.append(el)
    return dict(f=out_f, w=out_w, D=out_D, ell=out_ell, loss=loss, grads=np.array(grads))


@pytest.mark.parametrize("seed,stale", [(10, True), (11, False), (12, True)])
def test_whole_pass_matches_scalar_reimplementation(seed, stale):
    c = _tiny_case(seed, stale=stale)
    hp = dict(alpha=1.3, beta=0.6, xi=0.2, lam=0.4)
    res = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"],
                                c["lag"], grad_scale=1.7, **hp)
    ref = _scalar_reimplementation(c, hp["alpha"], hp["beta"], hp["xi"], hp["lam"], 1.7)
    np.testing.assert_allclose(res["freshness"], ref["f"], rtol=1e-13, atol=0)
    np.testing.assert_allclose(res["weights"], ref["w"], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(res["D_roll"], ref["D"], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(res["ell"], ref["ell"], rtol=1e-12, atol=1e-16)
    assert abs(res["loss"] - ref["loss"]) < 1e-14
    np.testing.assert_allclose(res["dlogits_exact"], ref["grads"], rtol=1e-11, atol=1e-16)
    assert res["freshness"][1] == 0.0 and res["cover"][1] == 0.0          # the empty sample
    assert np.any(res["weights"] == 0.0) and np.any(res["weights"] > 0.0)  # both branches taken
    np.testing.assert_allclose(res["agg"][0], np.mean(res["freshness"]), rtol=1e-15)
    np.testing.assert_allclose(res["agg"][1], np.mean(res["cover"]), rtol=1e-15)


def test_fresh_buffer_gives_unit_ratio_and_unit_score():
    c = _tiny_case(20, stale=False, lag=(0, 0, 0, 0))
    _, lp = orc.token_logprobs(c["z"], c["y"], c["mask"])
    res = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], lp, c["lq"], None, c["seq"], c["lag"],
                                alpha=2.0, beta=3.0, xi=0.0, lam=0.5)
    assert np.all(res["rho"][c["mask"] == 1] == 1.0)
    assert np.all(res["D_roll"] == 0.0) and np.all(res["D_sup"] == 0.0)
    valid = res["n_train"] > 0
    assert np.all(res["freshness"][valid] == 1.0) and np.all(res["freshness"][~valid] == 0.0)
    # with zero drift the anchor contributes nothing: loss is the weighted mean of l_i
    assert abs(res["loss"] - float(np.sum(res["weights"] * res["ell"])) / 4) < 1e-15


def test_gradient_rows_sum_to_zero_gated_rows_exactly_zero():
    c = _tiny_case(21, lag=(0, 1, 40, 2))
    res = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"],
                                c["lag"], alpha=1.0, beta=1.0, xi=0.05, lam=0.1)
    g = res["dlogits_exact"]
    assert np.max(np.abs(g.sum(axis=1))) < 1e-15
    cu = res["cu_seqlens"]
    assert res["weights"][2] == 0.0 and res["freshness"][2] > 0.0         # lag 40 -> gated
    assert np.all(g[cu[2]:cu[3]] == 0.0) and np.all(res["dlogits"][cu[2]:cu[3]] == 0.0)
    assert np.all(g[c["mask"] == 0] == 0.0)
    live = (c["mask"] == 1) & (np.repeat(res["weights"], c["seq"]) > 0)
    assert np.all(np.abs(g[live]).sum(axis=1) > 0)
    # gating removes the sample from the loss but not from the 1/B normaliser
    keep = [0, 3]
    L = sum(res["weights"][i] * (res["ell"][i] + 0.1 * res["D_roll"][i]) for i in keep) / 4
    assert abs(res["loss"] - L) < 1e-15


def test_gradient_by_finite_differences_of_surrogate():
    """F(z) = sum_t m_t w_i/(B n_i) [ (lp_t - lq_t)^2 / 2 + lambda k(lp_t - lb_t) ] with w frozen
    has dF/dlp = (lp - lq) + lambda rho delta = -(A - lambda rho delta): the oracle's gradient
    must equal grad F.  log-softmax here comes from scipy, not from the oracle."""
    c = _tiny_case(22, V=6, seq=(2, 3), lag=(1, 0))
    c["mask"][:] = 1
    c["mask"][3] = 0
    hp = dict(alpha=0.8, beta=0.3, xi=0.1, lam=0.7)
    res = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"],
                                c["lag"], grad_scale=2.5, **hp)
    w, n, cu = res["weights"], res["n_train"], res["cu_seqlens"]
    T, V = c["z"].shape
    B = 2
    sample_of = np.repeat(np.arange(B), c["seq"])

    def F(zz):
        lp = scipy.special.log_softmax(zz, axis=1)[np.arange(T), c["y"]]
        tot = 0.0
        for t in range(T):
            if not c["mask"][t]:
                continue
            i = sample_of[t]
            d = lp[t] - c["lb"][t]
            tot += 2.5 * w[i] / (B * n[i]) * (0.5 * (lp[t] - c["lq"][t]) ** 2
                                             + hp["lam"] * (math.exp(d) * d - math.exp(d) + 1))
        return tot

    h = 1e-6
    num = np.zeros((T, V))
    for t, v in itertools.product(range(T), range(V)):
        zp, zm = c["z"].copy(), c["z"].copy()
        zp[t, v] += h
        zm[t, v] -= h
        num[t, v] = (F(zp) - F(zm)) / (2 * h)
    scale = np.max(np.abs(num))
    assert scale > 1e-3
    assert np.max(np.abs(num - res["dlogits_exact"])) < 1e-6 * scale * 10
    assert np.all(res["dlogits_exact"][3] == 0.0)


def test_sequence_lengths_must_cover_all_rows():
    c = _tiny_case(23)
    with pytest.raises(ValueError):
        orc.fopd_loss_fwd_bwd(c["z"][:-1], c["y"][:-1], c["mask"][:-1], c["lb"][:-1], c["lq"][:-1],
                              None, c["seq"], c["lag"], 1.0, 1.0, 0.0, 0.0)


# ---------------------------------------------------------------------------------------
# rounding to the storage types
# ---------------------------------------------------------------------------------------

def test_bf16_rounding_matches_library_on_float32_inputs():
    rng = _rng(7)
    x32 = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 1e-6, 5000),
                          rng.normal(0, 1e30, 5000), [0.0, -0.0, 1.0, -1.0, 3.3895313892515355e38],
                          rng.normal(0, 1e-39, 2000)]).astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_to_bf16(x32.astype(np.float64))
    assert np.array_equal(got, want)


def test_bf16_rounding_ties_and_no_double_rounding():
    e = 2.0 ** -7                                  # bf16 spacing in [1, 2)
    assert orc.round_to_bf16(1.0 + e / 2) == 1.0            # tie -> even (mantissa 0)
    assert orc.round_to_bf16(1.0 + 3 * e / 2) == 1.0 + 2 * e  # tie -> even (mantissa 2)
    x = 1.0 + e / 2 + 2.0 ** -40                   # just above the tie; float32 would lose the 2^-40
    assert np.float64(np.float32(x)) == 1.0 + e / 2
    assert orc.round_to_bf16(x) == 1.0 + e
    assert orc.round_to_bf16(-x) == -(1.0 + e)
    np.testing.assert_array_equal(orc.bf16_ulp([1.0, 1.99, 2.0, 0.75, 0.0]),
                                  [e, e, 2 * e, e / 2, 2.0 ** -133])


# ---------------------------------------------------------------------------------------
# full-vocabulary rollout drift (Eq. kl-diagnostics as printed)
# ---------------------------------------------------------------------------------------

def test_full_kl_matches_library_pinsker_and_sampled_estimator():
    import scipy.stats
    rng = _rng(40)
    T, V = 7, 60
    z = rng.normal(0, 2, size=(T, V))
    zs = z + rng.normal(0, 0.4, size=(T, V))
    zs[3] = z[3] + 1.75                         # a constant shift is the same distribution
    mask = np.array([1, 1, 1, 1, 0, 1, 1], dtype=np.uint8)
    kl, lse, lse_s = orc.rollout_kl_full(z, zs, mask)
    p = scipy.special.softmax(z, axis=1)
    q = scipy.special.softmax(zs, axis=1)
    ref = scipy.stats.entropy(p, q, axis=1)     # library KL(p || q)
    live = mask == 1
    np.testing.assert_allclose(kl[live], ref[live], rtol=1e-11, atol=1e-15)
    rev = scipy.stats.entropy(q, p, axis=1)
    assert np.max(np.abs(kl[live] - rev[live])[[0, 1, 2]]) > 1e-4       # direction: current || stale
    assert kl[4] == 0.0 and abs(kl[3]) < 1e-14 and np.all(kl[live] >= -1e-15)
    tv = 0.5 * np.abs(p - q).sum(axis=1)
    assert np.all(tv[live] <= np.sqrt(kl[live] / 2) + 1e-12)           # Pinsker
    np.testing.assert_allclose(lse[live], scipy.special.logsumexp(z, axis=1)[live], rtol=1e-14)
    np.testing.assert_allclose(lse_s[live], scipy.special.logsumexp(zs, axis=1)[live], rtol=1e-14)
    # the sampled-token estimator used by the default path has this KL as its mean under the stale policy
    logp, logq = np.log(p), np.log(q)
    for t in (0, 5):
        est = sum(q[t, y] * orc.kl_estimator(logp[t, y] - logq[t, y]) for y in range(V))
        assert abs(est - kl[t]) < 1e-12


def test_full_kl_gradient_by_finite_differences():
    """F(z) = sum_t m_t w_i/(B n_i) [ (lp_t - lq_t)^2 / 2 + lambda KL(softmax(z_t) || softmax(z'_t)) ], w frozen."""
    rng = _rng(41)
    seq = np.array([3, 2], dtype=np.int32)
    T, V, B = 5, 6, 2
    z = rng.normal(0, 1.5, size=(T, V))
    zs = z + rng.normal(0, 0.5, size=(T, V))
    y = rng.integers(0, V, size=T).astype(np.int32)
    mask = np.array([1, 1, 0, 1, 1], dtype=np.uint8)
    lq = scipy.special.log_softmax(z, axis=1)[np.arange(T), y] + rng.normal(-0.3, 0.4, T)
    lag = np.array([1, 0], dtype=np.int32)
    hp = dict(alpha=0.9, beta=0.0, xi=0.05, lam=0.8)
    res = orc.fopd_loss_fwd_bwd_full_kl(z, zs, y, mask, lq, None, seq, lag, grad_scale=1.5, **hp)
    w, n = res["weights"], res["n_train"]
    sample_of = np.repeat(np.arange(B), seq)
    assert np.all(w > 0)
    np.testing.assert_allclose(res["D_roll"][0], np.mean(res["roll_kl"][[0, 1]]), rtol=1e-14)   # masked row 2 left out

    def F(zz):
        logp_all = scipy.special.log_softmax(zz, axis=1)
        logq_all = scipy.special.log_softmax(zs, axis=1)
        tot = 0.0
        for t in range(T):
            if not mask[t]:
                continue
            i = sample_of[t]
            kl_t = float(np.sum(np.exp(logp_all[t]) * (logp_all[t] - logq_all[t])))
            tot += 1.5 * w[i] / (B * n[i]) * (0.5 * (logp_all[t, y[t]] - lq[t]) ** 2 + hp["lam"] * kl_t)
        return tot

    h = 1e-6
    num = np.zeros((T, V))
    for t, v in itertools.product(range(T), range(V)):
        zp, zm = z.copy(), z.copy()
        zp[t, v] += h
        zm[t, v] -= h
        num[t, v] = (F(zp) - F(zm)) / (2 * h)
    scale = np.max(np.abs(num))
    assert np.max(np.abs(num - res["dlogits_exact"])) < 1e-5 * scale
    assert np.all(res["dlogits_exact"][2] == 0.0) and np.max(np.abs(res["dlogits_exact"].sum(axis=1))) < 1e-15
    # lambda = 0 reduces to the default path's gradient with no anchor
    r0 = orc.fopd_loss_fwd_bwd_full_kl(z, zs, y, mask, lq, None, seq, lag, 0.0, 0.0, 0.05, 0.0)
    lb = scipy.special.log_softmax(z, axis=1)[np.arange(T), y]
    r1 = orc.fopd_loss_fwd_bwd(z, y, mask, lb, lq, None, seq, lag, 0.0, 0.0, 0.05, 0.0)
    np.testing.assert_allclose(r0["dlogits_exact"], r1["dlogits_exact"], rtol=1e-13, atol=1e-18)
    assert abs(r0["loss"] - r1["loss"]) < 1e-15


# ---------------------------------------------------------------------------------------
# invariances of the whole pass
# ---------------------------------------------------------------------------------------

def test_invariances_shift_vocabulary_permutation_sample_permutation_scale():
    c = _tiny_case(50, V=13, seq=(4, 3, 5), lag=(0, 2, 1))
    hp = dict(alpha=1.1, beta=0.4, xi=0.1, lam=0.3)

    def run(z, y, seq=None, order=None, g=1.0):
        cc = dict(c)
        if order is not None:                    # reorder whole samples
            starts = np.concatenate([[0], np.cumsum(c["seq"])])
            rows = np.concatenate([np.arange(starts[i], starts[i + 1]) for i in order])
            cc = {k: (v[rows] if isinstance(v, np.ndarray) and v.shape[:1] == (len(c["y"]),) else v) for k, v in c.items()}
            z, y = z[rows], y[rows]
            cc["seq"], cc["lag"] = c["seq"][list(order)], c["lag"][list(order)]
        return orc.fopd_loss_fwd_bwd(z, y, cc["mask"], cc["lb"], cc["lq"], cc["lqs"], cc["seq"], cc["lag"],
                                     grad_scale=g, **hp)

    base = run(c["z"], c["y"])
    assert np.all(base["freshness"] > 0) and np.all(base["freshness"] <= 1)
    # (1) adding a constant to a row's logits changes nothing but lse
    shift = _rng(51).normal(0, 30, size=(len(c["y"]), 1))
    sh = run(c["z"] + shift, c["y"])
    np.testing.assert_allclose(sh["logp"], base["logp"], atol=1e-12)
    np.testing.assert_allclose(sh["dlogits_exact"], base["dlogits_exact"], atol=1e-14)
    assert abs(sh["loss"] - base["loss"]) < 1e-13
    # (2) relabelling the vocabulary permutes the gradient columns
    perm = _rng(52).permutation(13)
    inv = np.argsort(perm)
    pv = run(c["z"][:, perm], inv[c["y"]].astype(np.int32))
    np.testing.assert_allclose(pv["dlogits_exact"], base["dlogits_exact"][:, perm], atol=1e-15)
    np.testing.assert_allclose(pv["freshness"], base["freshness"], rtol=1e-13)
    # (3) reordering the samples reorders the per-sample outputs and leaves the loss alone
    order = (2, 0, 1)
    ro = run(c["z"], c["y"], order=order)
    np.testing.assert_allclose(ro["freshness"], base["freshness"][list(order)], rtol=1e-14)
    assert abs(ro["loss"] - base["loss"]) < 1e-15
    # (4) the upstream scale multiplies the gradient and nothing else
    sc = run(c["z"], c["y"], g=-3.5)
    np.testing.assert_allclose(sc["dlogits_exact"], -3.5 * base["dlogits_exact"], rtol=1e-14, atol=1e-300)
    assert sc["loss"] == base["loss"]


def test_full_teacher_variant_gradient_and_link_to_sampled_form():
    """Distribution-level token loss KL(pi_theta || teacher): finite differences of
    F(z) = sum_t m_t w_i/(B n_i) [ KL(softmax(z_t) || q_t) + lambda k(lp_t - lb_t) ] (w frozen), and the
    on-policy identity: averaging the default path's sampled-token gradient over y ~ softmax(z) gives
    this variant's KL gradient."""
    rng = _rng(60)
    seq = np.array([2, 3], dtype=np.int32)
    T, V, B = 5, 7, 2
    z = rng.normal(0, 1.3, size=(T, V))
    zq = rng.normal(0, 1.3, size=(T, V))
    y = rng.integers(0, V, size=T).astype(np.int32)
    mask = np.array([1, 1, 1, 0, 1], dtype=np.uint8)
    lb = scipy.special.log_softmax(z, axis=1)[np.arange(T), y] + rng.normal(0, 0.3, T)
    lag = np.array([0, 1], dtype=np.int32)
    hp = dict(alpha=0.7, beta=0.0, xi=0.02, lam=0.6)
    res = orc.fopd_loss_fwd_bwd_full_teacher(z, zq, y, mask, lb, None, seq, lag, grad_scale=0.8, **hp)
    w, n = res["weights"], res["n_train"]
    sample_of = np.repeat(np.arange(B), seq)
    logq_all = scipy.special.log_softmax(zq, axis=1)
    np.testing.assert_allclose(res["teacher_logp"][mask == 1], logq_all[np.arange(T), y][mask == 1], atol=1e-13)
    np.testing.assert_allclose(res["ell"][0], np.mean(res["token_kl"][:2]), rtol=1e-14)

    def F(zz):
        logp_all = scipy.special.log_softmax(zz, axis=1)
        tot = 0.0
        for t in range(T):
            if not mask[t]:
                continue
            i = sample_of[t]
            d = logp_all[t, y[t]] - lb[t]
            kl_t = float(np.sum(np.exp(logp_all[t]) * (logp_all[t] - logq_all[t])))
            tot += 0.8 * w[i] / (B * n[i]) * (kl_t + hp["lam"] * (math.exp(d) * d - math.exp(d) + 1))
        return tot

    h = 1e-6
    num = np.zeros((T, V))
    for t, v in itertools.product(range(T), range(V)):
        zp, zm = z.copy(), z.copy()
        zp[t, v] += h
        zm[t, v] -= h
        num[t, v] = (F(zp) - F(zm)) / (2 * h)
    assert np.max(np.abs(num - res["dlogits_exact"])) < 1e-5 * np.max(np.abs(num))
    assert np.all(res["dlogits_exact"][3] == 0.0)
    # on-policy link, one row, no anchor: E_{y ~ p}[ A_y (p - e_y) ] with A_y = log q_y - log p_y
    t = 0
    lse_t = scipy.special.logsumexp(z[t])
    p = np.exp(z[t] - lse_t)
    mean_sampled = sum(p[v] * orc.dlogits_row(z[t], v, lse_t, logq_all[t, v] - (z[t, v] - lse_t)) for v in range(V))
    kl_t = float(np.sum(p * ((z[t] - lse_t) - logq_all[t])))
    full = orc.dlogits_row_full_kl(z[t], zq[t], 0, lse_t, scipy.special.logsumexp(zq[t]), kl_t, 0.0, 1.0)
    np.testing.assert_allclose(mean_sampled, full, atol=1e-14)


# ---------------------------------------------------------------------------------------
# logits made from hidden states (the projection in front of the pass)
# ---------------------------------------------------------------------------------------

def test_projection_by_integer_brute_force_and_special_cases():
    rs = _rng(41)
    T, d, V = 3, 4, 5                                   # all different: a transposed operand cannot pass
    hidden = rs.integers(-3, 4, size=(T, d))
    weight = rs.integers(-3, 4, size=(V, d))
    z = orc.lm_head_logits(hidden, weight)
    assert z.shape == (T, V)
    for t in range(T):
        for v in range(V):
            exact = sum(int(hidden[t, k]) * int(weight[v, k]) for k in range(d))    # Python ints
            assert z[t, v] == float(exact)
    y = np.array([4, 0, 2])
    lse, lp = orc.lm_head_token_logprobs(hidden, weight, y, np.array([1, 0, 1]))
    for t in (0, 2):
        zs = [sum(int(hidden[t, k]) * int(weight[v, k]) for k in range(d)) for v in range(V)]
        ref = math.log(math.fsum(math.exp(a - max(zs)) for a in zs)) + max(zs)
        assert abs(lse[t] - ref) < 1e-13 and abs(lp[t] - (zs[y[t]] - ref)) < 1e-13
    assert lse[1] == 0.0 and lp[1] == 0.0
    # identity projection: the logits are the hidden states themselves
    h = rs.normal(size=(6, 7))
    yy = rs.integers(0, 7, size=6)
    a = orc.lm_head_token_logprobs(h, np.eye(7), yy)
    b = orc.token_logprobs(h, yy)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    # one more vector added to every vocabulary row shifts row t's logits by h_t . c: lp unchanged
    w = rs.normal(size=(9, 7))
    c = rs.normal(size=7)
    y9 = rs.integers(0, 9, size=6)
    l0, p0 = orc.lm_head_token_logprobs(h, w, y9)
    l1, p1 = orc.lm_head_token_logprobs(h, w + c[None, :], y9)
    np.testing.assert_allclose(p1, p0, atol=1e-13)
    np.testing.assert_allclose(l1 - l0, h @ c, atol=1e-13)
    with pytest.raises(ValueError):
        orc.lm_head_logits(np.zeros((2, 3)), np.zeros((3, 2)))


# ---------------------------------------------------------------------------------------
# two aligned sets: U^roll carries the rollout drift, U^sup the token loss and supervision drift
# ---------------------------------------------------------------------------------------

def _two_set_case(seed):
    c = _tiny_case(seed, V=9, seq=(6, 5, 4, 7, 3), lag=(0, 1, 2, 0, 1))
    rng = _rng(seed + 1000)
    c["mask"] = rng.integers(0, 4, size=len(c["mask"])).astype(np.uint8)      # 0 none, 1 both, 2 roll, 3 sup
    c["mask"][6:11] = np.array([3, 3, 0, 3, 3], dtype=np.uint8)              # sample 1: U^roll empty -> invalid
    c["mask"][11:15] = np.array([2, 0, 2, 2], dtype=np.uint8)               # sample 2: U^sup empty -> invalid
    c["mask"][0:6] = np.array([1, 2, 3, 0, 2, 2], dtype=np.uint8)           # sample 0: all four kinds
    return c


def _scalar_two_sets(c, alpha, beta, xi, lam, g):
    """Algorithm 1 with the two sets kept apart, in plain Python floats."""
    z, y, mask = c["z"], c["y"], c["mask"]
    T, V = z.shape
    B = len(c["seq"])
    k = lambda d: math.exp(d) * d - math.exp(d) + 1.0
    res = dict(f=[], w=[], Dr=[], Ds=[], ell=[], m_roll=[], m_sup=[], grads=[[0.0] * V for _ in range(T)], loss=0.0)
    start = 0
    for i in range(B):
        H = int(c["seq"][i])
        idx = range(start, start + H)
        start += H
        U_roll = [t for t in idx if mask[t] in (1, 2)]
        U_sup = [t for t in idx if mask[t] in (1, 3)]
        if not U_roll or not U_sup:                       # invalid-sample branch: f = 0, both ratios 0
            for key in ("f", "w", "Dr", "Ds", "ell", "m_roll", "m_sup"):
                res[key].append(0.0)
            continue
        lp, lse = {}, {}
        for t in set(U_roll) | set(U_sup):
            mx = max(float(v) for v in z[t])
            lse[t] = mx + math.log(sum(math.exp(float(v) - mx) for v in z[t]))
            lp[t] = float(z[t][y[t]]) - lse[t]
        Dr = sum(k(lp[t] - c["lb"][t]) for t in U_roll) / len(U_roll)
        Ds = sum(k(c["lq"][t] - c["lqs"][t]) for t in U_sup) / len(U_sup)
        el = sum(lp[t] - c["lq"][t] for t in U_sup) / len(U_sup)
        f = math.exp(-alpha * math.sqrt(Dr) - beta * math.sqrt(Ds)) / (int(c["lag"][i]) + 1)
        w = max(f - xi, 0.0)
        res["loss"] += w * (el + lam * Dr) / B
        for t in set(U_roll) | set(U_sup):
            ct = 0.0
            if t in U_sup:
                ct += (c["lq"][t] - lp[t]) / len(U_sup)
            if t in U_roll:
                d = lp[t] - c["lb"][t]
                ct -= lam * math.exp(d) * d / len(U_roll)
            ct *= g * w / B
            for v in range(V):
                res["grads"][t][v] = ct * (math.exp(float(z[t][v]) - lse[t]) - (1.0 if v == y[t] else 0.0))
        for key, val in (("f", f), ("w", w), ("Dr", Dr), ("Ds", Ds), ("ell", el),
                         ("m_roll", len(U_roll) / H), ("m_sup", len(U_sup) / H)):
            res[key].append(val)
    res["grads"] = np.array(res["grads"])
    return res


@pytest.mark.parametrize("seed", [30, 31])
def test_two_aligned_sets_against_scalar_reimplementation(seed):
    c = _two_set_case(seed)
    hp = dict(alpha=0.9, beta=1.4, xi=0.1, lam=0.6)
    res = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"], c["lag"],
                                grad_scale=0.7, **hp)
    ref = _scalar_two_sets(c, hp["alpha"], hp["beta"], hp["xi"], hp["lam"], 0.7)
    np.testing.assert_allclose(res["freshness"], ref["f"], rtol=1e-13, atol=0)
    np.testing.assert_allclose(res["weights"], ref["w"], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(res["D_roll"], ref["Dr"], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(res["D_sup"], ref["Ds"], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(res["ell"], ref["ell"], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(res["cover"], ref["m_sup"], rtol=1e-15)
    np.testing.assert_allclose(res["cover_roll"], ref["m_roll"], rtol=1e-15)
    assert abs(res["loss"] - ref["loss"]) < 1e-14
    np.testing.assert_allclose(res["dlogits_exact"], ref["grads"], rtol=1e-11, atol=1e-16)
    # either set empty: invalid, whatever the other holds (Algorithm 1)
    assert res["freshness"][1] == 0.0 and res["freshness"][2] == 0.0
    assert res["cover"][1] == 0.0 and res["cover_roll"][2] == 0.0
    assert not np.any(res["dlogits_exact"][6:15])
    # the two coverage means are different numbers now
    np.testing.assert_allclose(res["agg"][1], np.mean(ref["m_roll"]), rtol=1e-15)
    np.testing.assert_allclose(res["agg"][2], np.mean(ref["m_sup"]), rtol=1e-15)
    assert res["cover_roll"][0] == 4 / 6 and res["cover"][0] == 2 / 6
    # a row in U^roll only has a gradient from the anchor alone; with lambda = 0 it is exactly zero
    res0 = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"], c["lag"],
                                 alpha=0.9, beta=1.4, xi=0.1, lam=0.0)
    assert np.any(res["dlogits_exact"][1]) and not np.any(res0["dlogits_exact"][1])
    assert np.any(res0["dlogits_exact"][2])                # a U^sup-only row (row 2) keeps the loss term
    # an invalid sample has weight 0 whatever the threshold is, also a negative one
    resn = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"], c["lag"],
                                 alpha=0.9, beta=1.4, xi=-0.5, lam=0.6)
    assert resn["weights"][1] == 0.0 and resn["weights"][2] == 0.0 and resn["weights"][0] > 0.5
    assert not np.any(resn["dlogits_exact"][6:15])


def test_two_aligned_sets_plain_mask_means_both_and_counts():
    c = _two_set_case(33)
    cu = orc.segment_offsets(c["seq"])
    n_sup, n_roll = orc.trainable_counts(c["mask"], cu), orc.roll_counts(c["mask"], cu)
    start = 0
    for i, H in enumerate(c["seq"]):
        seg = [int(m) for m in c["mask"][start:start + int(H)]]
        start += int(H)
        assert n_sup[i] == sum(1 for m in seg if m in (1, 3)) and n_roll[i] == sum(1 for m in seg if m in (1, 2))
    # a 0/1 mask (and any other non-zero byte) puts a row in both sets
    both = (c["mask"] != 0).astype(np.uint8)
    odd = both * 255
    assert np.array_equal(orc.trainable_counts(both, cu), orc.roll_counts(both, cu))
    assert np.array_equal(orc.trainable_counts(odd, cu), orc.trainable_counts(both, cu))
    assert np.array_equal(orc.roll_counts(odd, cu), orc.roll_counts(both, cu))


def test_two_aligned_sets_gradient_by_finite_differences():
    c = _two_set_case(34)
    T, V = c["z"].shape
    hp = dict(alpha=0.5, beta=0.5, xi=0.02, lam=0.8)
    res = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"], c["lag"], **hp)
    w, B = res["weights"], len(c["seq"])
    cu = orc.segment_offsets(c["seq"])
    n_sup, n_roll = orc.trainable_counts(c["mask"], cu), orc.roll_counts(c["mask"], cu)
    sample_of = np.repeat(np.arange(B), c["seq"])

    def F(zz):
        """Surrogate with the weights frozen: its gradient is the method's semi-gradient."""
        lp_all = scipy.special.log_softmax(zz, axis=1)
        tot = 0.0
        for t in range(T):
            i = sample_of[t]
            if w[i] == 0.0:
                continue
            lp = lp_all[t, c["y"][t]]
            if c["mask"][t] in (1, 3):
                tot += w[i] / (B * n_sup[i]) * 0.5 * (lp - c["lq"][t]) ** 2
            if c["mask"][t] in (1, 2):
                d = lp - c["lb"][t]
                tot += w[i] / (B * n_roll[i]) * hp["lam"] * (math.exp(d) * d - math.exp(d) + 1.0)
        return tot

    h = 1e-6
    num = np.zeros((T, V))
    for t, v in itertools.product(range(T), range(V)):
        zp, zm = c["z"].copy(), c["z"].copy()
        zp[t, v] += h
        zm[t, v] -= h
        num[t, v] = (F(zp) - F(zm)) / (2 * h)
    assert np.max(np.abs(num - res["dlogits_exact"])) < 1e-6 * np.max(np.abs(num))


def test_unit_rows_are_the_gradient_of_the_sample_terms_and_scale_to_the_full_gradient():
    """Gradient rows at unit sample weight (the weight is a constant of the sample in the semi-gradient):
    (a) they are the finite-difference gradient of G(z) = g/B sum over valid samples of (l_i-surrogate + lambda
    D_i^roll), written here with scipy's log-softmax and no weight at all; (b) weight x unit row is the full
    gradient row, also for gated samples (unit row non-zero, product zero); (c) an invalid sample has zero rows."""
    c = _two_set_case(36)
    T, V = c["z"].shape
    hp = dict(alpha=0.5, beta=0.5, xi=0.5, lam=0.8)             # gates the sample with lag 1
    res = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"], c["lag"],
                                grad_scale=1.7, unit_rows=True, **hp)
    B = len(c["seq"])
    cu = orc.segment_offsets(c["seq"])
    n_sup, n_roll = orc.trainable_counts(c["mask"], cu), orc.roll_counts(c["mask"], cu)
    sample_of = np.repeat(np.arange(B), c["seq"])

    def G(zz):
        lp_all = scipy.special.log_softmax(zz, axis=1)
        tot = 0.0
        for t in range(T):
            i = sample_of[t]
            if n_sup[i] == 0 or n_roll[i] == 0:
                continue
            lp = lp_all[t, c["y"][t]]
            if c["mask"][t] in (1, 3):
                tot += 1.7 / (B * n_sup[i]) * 0.5 * (lp - c["lq"][t]) ** 2
            if c["mask"][t] in (1, 2):
                d = lp - c["lb"][t]
                tot += 1.7 / (B * n_roll[i]) * hp["lam"] * (math.exp(d) * d - math.exp(d) + 1.0)
        return tot

    h = 1e-6
    num = np.zeros((T, V))
    for t, v in itertools.product(range(T), range(V)):
        zp, zm = c["z"].copy(), c["z"].copy()
        zp[t, v] += h
        zm[t, v] -= h
        num[t, v] = (G(zp) - G(zm)) / (2 * h)
    u = res["unit_rows_exact"]
    assert np.max(np.abs(num)) > 1e-3 and np.max(np.abs(num - u)) < 1e-6 * np.max(np.abs(num))
    w_rows = np.repeat(res["weights"], c["seq"])[:, None]
    np.testing.assert_allclose(w_rows * u, res["dlogits_exact"], rtol=1e-14, atol=0.0)
    gated = [i for i in range(B) if res["weights"][i] == 0.0 and min(n_sup[i], n_roll[i]) > 0]
    live = [i for i in range(B) if res["weights"][i] > 0.0]
    invalid = [i for i in range(B) if min(n_sup[i], n_roll[i]) == 0]
    assert gated and live and invalid                                 # the case holds all three kinds
    for i in gated:
        assert np.any(u[cu[i]:cu[i + 1]] != 0.0) and np.all(res["dlogits_exact"][cu[i]:cu[i + 1]] == 0.0)
    for i in invalid:
        assert np.all(u[cu[i]:cu[i + 1]] == 0.0)
    assert np.array_equal(res["unit_rows"], orc.round_to_f32(u))


def test_two_aligned_sets_in_the_two_tensor_variants():
    """Full-vocabulary drift and distribution-level loss with the sets apart: D^roll over U^roll, the
    token loss over U^sup, checked against the definitions evaluated with scipy."""
    c = _two_set_case(35)
    rng = _rng(77)
    T, V = c["z"].shape
    z2 = c["z"] + rng.normal(0, 0.3, size=(T, V))
    cu = orc.segment_offsets(c["seq"])
    lp_all = scipy.special.log_softmax(c["z"], axis=1)
    l2_all = scipy.special.log_softmax(z2, axis=1)
    kl_rows = np.sum(np.exp(lp_all) * (lp_all - l2_all), axis=1)
    res = orc.fopd_loss_fwd_bwd_full_kl(c["z"], z2, c["y"], c["mask"], c["lq"], c["lqs"], c["seq"], c["lag"],
                                        0.7, 0.7, 0.0, 0.5)
    rest = orc.fopd_loss_fwd_bwd_full_teacher(c["z"], z2, c["y"], c["mask"], c["lb"], c["lqs"], c["seq"], c["lag"],
                                              0.7, 0.7, 0.0, 0.5)
    for i in (0, 3, 4):
        rows = range(int(cu[i]), int(cu[i + 1]))
        U_roll = [t for t in rows if c["mask"][t] in (1, 2)]
        U_sup = [t for t in rows if c["mask"][t] in (1, 3)]
        if not U_roll or not U_sup:
            continue
        np.testing.assert_allclose(res["D_roll"][i], np.mean(kl_rows[U_roll]), rtol=1e-12)
        np.testing.assert_allclose(rest["ell"][i], np.mean(kl_rows[U_sup]), rtol=1e-12)
    assert res["freshness"][1] == 0.0 and rest["freshness"][2] == 0.0
    # coefficient supports: the advantage part lives on U^sup, the full-KL part on U^roll
    assert np.all((res["c1"] != 0) <= np.isin(c["mask"], (1, 3))) and np.all((res["c2"] != 0) <= np.isin(c["mask"], (1, 2)))
    assert np.all((rest["c2"] != 0) <= np.isin(c["mask"], (1, 3))) and np.all((rest["c1"] != 0) <= np.isin(c["mask"], (1, 2)))


def test_two_aligned_sets_two_tensor_gradients_by_finite_differences():
    c = _two_set_case(36)
    rng = _rng(78)
    T, V = c["z"].shape
    z2 = c["z"] + rng.normal(0, 0.3, size=(T, V))
    B = len(c["seq"])
    cu = orc.segment_offsets(c["seq"])
    n_sup, n_roll = orc.trainable_counts(c["mask"], cu), orc.roll_counts(c["mask"], cu)
    sample_of = np.repeat(np.arange(B), c["seq"])
    l2_all = scipy.special.log_softmax(z2, axis=1)
    lam = 0.6
    kl = orc.fopd_loss_fwd_bwd_full_kl(c["z"], z2, c["y"], c["mask"], c["lq"], c["lqs"], c["seq"], c["lag"],
                                       0.4, 0.4, 0.01, lam, grad_scale=1.3)
    te = orc.fopd_loss_fwd_bwd_full_teacher(c["z"], z2, c["y"], c["mask"], c["lb"], c["lqs"], c["seq"], c["lag"],
                                            0.4, 0.4, 0.01, lam, grad_scale=1.3)

    def surrogate(zz, w, teacher):
        lp_all = scipy.special.log_softmax(zz, axis=1)
        tot = 0.0
        for t in range(T):
            i = sample_of[t]
            if w[i] == 0.0:
                continue
            lp = lp_all[t, c["y"][t]]
            full = float(np.sum(np.exp(lp_all[t]) * (lp_all[t] - l2_all[t])))
            if c["mask"][t] in (1, 3):                        # token loss on U^sup
                tot += 1.3 * w[i] / (B * n_sup[i]) * (full if teacher else 0.5 * (lp - c["lq"][t]) ** 2)
            if c["mask"][t] in (1, 2):                        # anchor on U^roll
                d = lp - c["lb"][t]
                tot += 1.3 * w[i] / (B * n_roll[i]) * lam * ((math.exp(d) * d - math.exp(d) + 1.0) if teacher else full)
        return tot

    h = 1e-6
    for res, teacher in ((kl, False), (te, True)):
        num = np.zeros((T, V))
        for t, v in itertools.product(range(T), range(V)):
            zp, zm = c["z"].copy(), c["z"].copy()
            zp[t, v] += h
            zm[t, v] -= h
            num[t, v] = (surrogate(zp, res["weights"], teacher) - surrogate(zm, res["weights"], teacher)) / (2 * h)
        assert np.max(np.abs(num - res["dlogits_exact"])) < 2e-6 * np.max(np.abs(num)), teacher


# ---------------------------------------------------------------------------------------
# gradient carried through the output projection
# ---------------------------------------------------------------------------------------

def _projection_case(seed, T_seq=(3, 4), d=5, V=7):
    rng = _rng(seed)
    seq = np.array(T_seq, dtype=np.int32)
    T = int(seq.sum())
    H = rng.normal(0, 1.0, size=(T, d))
    W = rng.normal(0, 0.8, size=(V, d))
    y = rng.integers(0, V, size=T).astype(np.int32)
    mask = np.array([1, 2, 3, 1, 0, 1, 3][:T], dtype=np.uint8)
    lp = scipy.special.log_softmax(H @ W.T, axis=1)[np.arange(T), y]
    lb = lp + rng.normal(0, 0.3, T)
    lq = np.minimum(lp + rng.normal(-0.3, 0.5, T), 0.0)
    return dict(H=H, W=W, y=y, mask=mask, lb=lb, lq=lq, seq=seq, lag=np.array([0, 2], dtype=np.int32),
                f=np.array([0.8, 0.3]))


def test_projection_gradient_by_finite_differences_through_hidden_and_weight():
    """dL/dhidden and dL/dweight of the surrogate whose logits-gradient is the method's semi-gradient
    (weights and advantage frozen), by central differences through the projection: fixes which operand each
    contraction takes, along which axis, and that the three dimensions are not mixed up (T, d, V all differ)."""
    c = _projection_case(3)
    xi, lam, g = 0.05, 0.7, 1.3
    res = orc.lm_head_loss_fwd_bwd(c["H"], c["W"], c["y"], c["mask"], c["lb"], c["lq"], c["seq"], c["lag"], c["f"],
                                   xi, lam, g)
    T, d = c["H"].shape
    V = c["W"].shape[0]
    assert res["dhidden_exact"].shape == (T, d) and res["dweight_exact"].shape == (V, d)
    wts, B = res["weights"], len(c["seq"])
    cu, n, nr = res["cu_seqlens"], res["n_train"], res["n_roll"]
    assert list(n) != list(nr)                                     # the two aligned sets differ in this case

    def surrogate(H, W):
        lpx = scipy.special.log_softmax(H @ W.T, axis=1)[np.arange(T), c["y"]]
        tot = 0.0
        for i in range(B):
            for t in range(int(cu[i]), int(cu[i + 1])):
                m = int(c["mask"][t])
                if m != 0 and m != 2:
                    tot += g * wts[i] / (B * int(n[i])) * 0.5 * (lpx[t] - c["lq"][t]) ** 2
                if m != 0 and m != 3:
                    dlt = lpx[t] - c["lb"][t]
                    tot += g * wts[i] / (B * int(nr[i])) * lam * (math.exp(dlt) * dlt - math.exp(dlt) + 1.0)
        return tot

    h = 1e-6
    for (t, k) in itertools.product(range(T), range(d)):
        Hp, Hm = c["H"].copy(), c["H"].copy()
        Hp[t, k] += h
        Hm[t, k] -= h
        fd = (surrogate(Hp, c["W"]) - surrogate(Hm, c["W"])) / (2 * h)
        assert abs(fd - res["dhidden_exact"][t, k]) <= 1e-8 + 1e-6 * abs(fd), (t, k)
    for (v, k) in itertools.product(range(V), range(d)):
        Wp, Wm = c["W"].copy(), c["W"].copy()
        Wp[v, k] += h
        Wm[v, k] -= h
        fd = (surrogate(c["H"], Wp) - surrogate(c["H"], Wm)) / (2 * h)
        assert abs(fd - res["dweight_exact"][v, k]) <= 1e-8 + 1e-6 * abs(fd), (v, k)
    assert np.any(res["dhidden_exact"][0] != 0.0) and not np.any(res["dhidden_exact"][4])   # row 4 is masked


def test_projection_gradient_reduces_to_the_stored_logits_pass_and_rounds_the_rows_once():
    """With the identity as the projection matrix the hidden states ARE the logits: dL/dhidden must be the
    bf16-rounded gradient rows of the stored-logits pass with the same supplied scores, and dL/dweight the
    outer-product sum of those rows with the hidden states (checked entry by entry with integer-valued rows)."""
    rng = _rng(8)
    V = 6
    seq = np.array([2, 3], dtype=np.int32)
    T = 5
    H = rng.integers(-3, 4, size=(T, V)).astype(np.float64)
    y = rng.integers(0, V, size=T).astype(np.int32)
    mask = np.ones(T, dtype=np.uint8)
    lp = scipy.special.log_softmax(H, axis=1)[np.arange(T), y]
    lb, lq = lp - 0.2, lp - 0.4
    f = np.array([0.9, 0.6])
    res = orc.lm_head_loss_fwd_bwd(H, np.eye(V), y, mask, lb, lq, seq, [0, 1], f, 0.1, 0.5, 2.0)
    # the stored-logits pass with weights f - xi: coefficient by hand for row 0 of sample 0 (n = 2, B = 2)
    c0 = 2.0 * (0.9 - 0.1) / (2 * 2) * ((lq[0] - lp[0]) - 0.5 * math.exp(lp[0] - lb[0]) * (lp[0] - lb[0]))
    row0 = c0 * (np.exp(H[0] - scipy.special.logsumexp(H[0])) - np.eye(V)[y[0]])
    np.testing.assert_allclose(res["dlogits_exact"][0], row0, rtol=1e-13, atol=1e-16)
    np.testing.assert_array_equal(res["dhidden"], res["dlogits"])          # identity projection
    np.testing.assert_array_equal(res["dlogits"], orc.round_to_bf16(res["dlogits_exact"]))
    for v in range(V):
        for k in range(V):
            want = math.fsum(float(res["dlogits"][t, v]) * float(H[t, k]) for t in range(T))
            assert abs(res["dweight"][v, k] - want) <= 1e-15
    assert abs(res["loss"] - ((0.8 * (0.4 + 0.5 * orc.kl_estimator(0.2)) + 0.5 * (0.4 + 0.5 * orc.kl_estimator(0.2))) / 2)) < 1e-14


# ---------------------------------------------------------------------------------------
# distribution-level token loss against a teacher stored as k tokens per row
# ---------------------------------------------------------------------------------------

def test_topk_teacher_hand_worked_rows():
    """The two rows of tests/golden/topk_teacher_hand_worked.txt: loss, per-token G and gradient literals worked by
    hand (slots out of vocabulary order; the floor of the rest binding in the second row)."""
    want = {}
    for line in open(os.path.join(GOLDEN, "topk_teacher_hand_worked.txt")):
        if line.strip() and not line.startswith("#"):
            name, *vals = line.split()
            want[name] = np.array([float(v) for v in vals])
    zA = np.log(np.array([4.0, 2.0, 1.0, 1.0]))
    ell, G = orc.topk_token_loss_row(zA, [1, 0], [math.log(0.5), math.log(0.25)], 1e-6)
    assert abs(ell - want["A_loss"][0]) < 1e-15
    np.testing.assert_allclose(G, want["A_G"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(orc.dlogits_row_topk(zA, 3, [1, 0], [math.log(0.5), math.log(0.25)], 1e-6, 0.0, 1.0),
                               want["A_grad"], rtol=0, atol=1e-15)
    zB = np.zeros(2)
    ell, G = orc.topk_token_loss_row(zB, [0], [0.0], 1.0 / 512.0)
    assert abs(ell - want["B_loss"][0]) < 1e-15
    np.testing.assert_allclose(G, want["B_G"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(orc.dlogits_row_topk(zB, 0, [0], [0.0], 1.0 / 512.0, 0.0, 1.0), want["B_grad"],
                               rtol=0, atol=1e-15)
    # the anchor's share of the row is the default path's: c1 (p - onehot)
    np.testing.assert_allclose(orc.dlogits_row_topk(zA, 3, [1, 0], [math.log(0.5), math.log(0.25)], 1e-6, 2.0, 0.0),
                               2.0 * (np.array([0.5, 0.25, 0.125, 0.125]) - np.array([0, 0, 0, 1.0])), atol=1e-15)


def test_topk_teacher_full_list_is_the_kl_and_coarsening_never_raises_it():
    """With every token listed the loss is KL(p || q) (scipy's rel_entr); merging tokens into the rest can only
    lower it (log-sum inequality), so nested lists give a non-decreasing sequence below the full KL; the order of
    the slots and unused slots (ids outside the vocabulary) do not matter; an empty list gives 0 and no gradient;
    a token listed twice is refused."""
    rng = _rng(91)
    V = 13
    for _ in range(6):
        z = rng.normal(0, 2.0, V)
        zq = rng.normal(0, 2.0, V)
        p = scipy.special.softmax(z)
        logq = scipy.special.log_softmax(zq)
        full = float(np.sum(scipy.special.rel_entr(p, np.exp(logq))))
        order = np.argsort(-logq)                       # the teacher's own ranking
        ell_all, G_all = orc.topk_token_loss_row(z, order, logq[order], 1e-12)
        assert abs(ell_all - full) < 1e-13
        np.testing.assert_allclose(G_all, scipy.special.log_softmax(z) - logq, atol=1e-13)
        prev = -1e-15
        for k in range(0, V + 1):
            ids = order[:k]
            ell, _ = orc.topk_token_loss_row(z, ids, logq[ids], 1e-12)
            assert prev - 1e-13 <= ell <= full + 1e-13, (k, ell, prev, full)
            prev = ell
        ids = order[:5]
        a, Ga = orc.topk_token_loss_row(z, ids, logq[ids], 1e-12)
        perm = rng.permutation(5)
        b, Gb = orc.topk_token_loss_row(z, ids[perm], logq[ids][perm], 1e-12)
        padded_ids = np.concatenate([[-1], ids[:2], [V], ids[2:], [V + 7]])
        padded_lq = np.concatenate([[-0.1], logq[ids][:2], [-0.2], logq[ids][2:], [0.0]])
        c, Gc = orc.topk_token_loss_row(z, padded_ids, padded_lq, 1e-12)
        assert abs(a - b) < 1e-14 and abs(a - c) < 1e-14
        np.testing.assert_allclose(Ga, Gb, atol=1e-14)
        np.testing.assert_allclose(Ga, Gc, atol=1e-14)
        e0, _ = orc.topk_token_loss_row(z, [-1, -1], [0.0, 0.0], 1e-12)
        assert abs(e0) < 1e-15
        assert np.max(np.abs(orc.dlogits_row_topk(z, 2, [-1, -1], [0.0, 0.0], 1e-12, 0.0, 1.0))) < 1e-15
    with pytest.raises(ValueError):
        orc.topk_token_loss_row(np.zeros(5), [1, 3, 1], [-1.0, -1.0, -1.0], 1e-6)


def test_topk_teacher_pass_by_finite_differences_and_per_sample_means():
    """Whole pass on two aligned sets: finite differences of
    F(z) = sum_t w_i g / B ( [t in U^sup] l_t(z_t) / |U^sup| + [t in U^roll] lambda k(lp_t - lb_t) / |U^roll| ),
    with l_t written here from scipy's softmax and explicit event sums (weights frozen); l_i is the mean of l_t over
    U^sup; D^sup comes from the two sampled-token teacher arrays and is 0 when either is missing."""
    c = _two_set_case(52)
    rng = _rng(53)
    T, V = c["z"].shape
    B = len(c["seq"])
    k = 4
    zq = c["z"] + rng.normal(0, 0.8, size=(T, V))
    logq_all = scipy.special.log_softmax(zq, axis=1)
    ids = np.argsort(-logq_all, axis=1)[:, :k].astype(np.int32)
    ids[1, 2] = -1                                      # an unused slot
    lq_list = np.take_along_axis(logq_all, np.maximum(ids, 0), axis=1)
    floor = 1e-4
    cu = orc.segment_offsets(c["seq"])
    n_sup, n_roll = orc.trainable_counts(c["mask"], cu), orc.roll_counts(c["mask"], cu)
    sample_of = np.repeat(np.arange(B), c["seq"])
    lam, g = 0.6, 1.3
    res = orc.fopd_loss_fwd_bwd_topk_teacher(c["z"], c["y"], c["mask"], c["lb"], ids, lq_list, floor, c["lq"],
                                             c["lqs"], c["seq"], c["lag"], 0.4, 0.4, 0.01, lam, grad_scale=g)
    assert np.any(res["weights"] > 0)

    def token_loss(zrow, t):
        p = scipy.special.softmax(zrow)
        listed = [int(u) for u in ids[t] if 0 <= u < V]
        tot, p_in, q_in = 0.0, 0.0, 0.0
        for j, u in enumerate(ids[t]):
            if 0 <= u < V:
                tot += p[u] * (math.log(p[u]) - lq_list[t, j])
                p_in += p[u]
                q_in += math.exp(lq_list[t, j])
        p_rest = sum(p[u] for u in range(V) if u not in listed)
        return tot + p_rest * (math.log(p_rest) - math.log(max(1.0 - q_in, floor)))

    for i in range(B):
        rows = [t for t in range(int(cu[i]), int(cu[i + 1])) if c["mask"][t] in (1, 3)]
        if n_sup[i] and n_roll[i]:
            assert abs(res["ell"][i] - sum(token_loss(c["z"][t], t) for t in rows) / len(rows)) < 1e-13
    ref = orc.fopd_loss_fwd_bwd(c["z"], c["y"], c["mask"], c["lb"], c["lq"], c["lqs"], c["seq"], c["lag"],
                                0.4, 0.4, 0.01, lam)
    np.testing.assert_allclose(res["D_sup"], ref["D_sup"], atol=1e-15)      # same sampled-token arrays
    np.testing.assert_allclose(res["D_roll"], ref["D_roll"], atol=1e-15)
    none = orc.fopd_loss_fwd_bwd_topk_teacher(c["z"], c["y"], c["mask"], c["lb"], ids, lq_list, floor, c["lq"], None,
                                              c["seq"], c["lag"], 0.4, 0.4, 0.01, lam)
    assert np.all(none["D_sup"] == 0.0) and np.any(ref["D_sup"] > 0.0)

    def surrogate(zz, w):
        lp_all = scipy.special.log_softmax(zz, axis=1)
        tot = 0.0
        for t in range(T):
            i = sample_of[t]
            if w[i] == 0.0:
                continue
            if c["mask"][t] in (1, 3):
                tot += g * w[i] / (B * n_sup[i]) * token_loss(zz[t], t)
            if c["mask"][t] in (1, 2):
                d = lp_all[t, c["y"][t]] - c["lb"][t]
                tot += g * w[i] / (B * n_roll[i]) * lam * (math.exp(d) * d - math.exp(d) + 1.0)
        return tot

    h = 1e-6
    num = np.zeros((T, V))
    for t, v in itertools.product(range(T), range(V)):
        zp, zm = c["z"].copy(), c["z"].copy()
        zp[t, v] += h
        zm[t, v] -= h
        num[t, v] = (surrogate(zp, res["weights"]) - surrogate(zm, res["weights"])) / (2 * h)
    assert np.max(np.abs(num - res["dlogits_exact"])) < 2e-6 * np.max(np.abs(num))
    # the loss value itself
    w = res["weights"]
    want = sum(w[i] * (res["ell"][i] + lam * res["D_roll"][i]) for i in range(B)) / B
    assert abs(res["loss"] - want) < 1e-15


def test_projection_with_listed_teacher_by_finite_differences_and_identity_projection():
    """The listed-teacher pass on projected logits: dL/dhidden and dL/dweight by central differences of the
    surrogate through the projection (weights frozen; T, d, V all different; two aligned sets; the token loss
    re-typed from scipy's softmax and explicit event sums), and the identity projection, under which the hidden
    states are the logits and dL/dhidden must be the stored-logits call's gradient rows."""
    c = _projection_case(8)
    rng = _rng(81)
    T, d = c["H"].shape
    V = c["W"].shape[0]
    k, floor = 3, 1e-3
    zq = c["H"] @ c["W"].T + rng.normal(0, 0.7, size=(T, V))
    logq_all = scipy.special.log_softmax(zq, axis=1)
    ids = np.argsort(-logq_all, axis=1)[:, :k].astype(np.int32)
    ids[2, 1] = V + 3                                   # an unused slot
    lq_list = np.take_along_axis(logq_all, np.minimum(ids, V - 1), axis=1)
    alpha, beta, xi, lam, g = 0.5, 0.0, 0.01, 0.7, 1.3
    res = orc.lm_head_loss_fwd_bwd_topk_teacher(c["H"], c["W"], c["y"], c["mask"], c["lb"], ids, lq_list, floor, None,
                                                None, c["seq"], c["lag"], alpha, beta, xi, lam, g)
    wts, B = res["weights"], len(c["seq"])
    cu, n, nr = res["cu_seqlens"], res["n_train"], res["n_roll"]
    assert np.all(wts > 0) and list(n) != list(nr)

    def token_loss(zrow, t):
        p = scipy.special.softmax(zrow)
        listed = [int(u) for u in ids[t] if 0 <= u < V]
        tot, q_in = 0.0, 0.0
        for j, u in enumerate(ids[t]):
            if 0 <= u < V:
                tot += p[u] * (math.log(p[u]) - lq_list[t, j])
                q_in += math.exp(lq_list[t, j])
        p_rest = sum(p[u] for u in range(V) if u not in listed)
        return tot + p_rest * (math.log(p_rest) - math.log(max(1.0 - q_in, floor)))

    def surrogate(H, W):
        z = H @ W.T
        lpx = scipy.special.log_softmax(z, axis=1)[np.arange(T), c["y"]]
        tot = 0.0
        for i in range(B):
            for t in range(int(cu[i]), int(cu[i + 1])):
                m = int(c["mask"][t])
                if m != 0 and m != 2:
                    tot += g * wts[i] / (B * int(n[i])) * token_loss(z[t], t)
                if m != 0 and m != 3:
                    dlt = lpx[t] - c["lb"][t]
                    tot += g * wts[i] / (B * int(nr[i])) * lam * (math.exp(dlt) * dlt - math.exp(dlt) + 1.0)
        return tot

    h = 1e-6
    for (t, j) in itertools.product(range(T), range(d)):
        Hp, Hm = c["H"].copy(), c["H"].copy()
        Hp[t, j] += h
        Hm[t, j] -= h
        fd = (surrogate(Hp, c["W"]) - surrogate(Hm, c["W"])) / (2 * h)
        assert abs(fd - res["dhidden_exact"][t, j]) <= 1e-8 + 1e-6 * abs(fd), (t, j)
    for (v, j) in itertools.product(range(V), range(d)):
        Wp, Wm = c["W"].copy(), c["W"].copy()
        Wp[v, j] += h
        Wm[v, j] -= h
        fd = (surrogate(c["H"], Wp) - surrogate(c["H"], Wm)) / (2 * h)
        assert abs(fd - res["dweight_exact"][v, j]) <= 1e-8 + 1e-6 * abs(fd), (v, j)
    assert not np.any(res["dhidden_exact"][4])                          # row 4 is in neither set
    # identity projection: hidden states are the logits
    z = c["H"] @ c["W"].T
    eye = np.eye(V)
    ident = orc.lm_head_loss_fwd_bwd_topk_teacher(z, eye, c["y"], c["mask"], c["lb"], ids, lq_list, floor, None, None,
                                                  c["seq"], c["lag"], alpha, beta, xi, lam, g)
    stored = orc.fopd_loss_fwd_bwd_topk_teacher(z, c["y"], c["mask"], c["lb"], ids, lq_list, floor, None, None, c["seq"],
                                                c["lag"], alpha, beta, xi, lam, grad_scale=g, out_dtype="bf16")
    np.testing.assert_array_equal(ident["dhidden"], stored["dlogits"])              # rounded once, bit for bit
    np.testing.assert_allclose(ident["dhidden_exact"], stored["dlogits_exact"], atol=1e-15)
    np.testing.assert_allclose(ident["dweight_exact"], stored["dlogits_exact"].T @ z, atol=1e-13)
    assert abs(ident["loss"] - stored["loss"]) < 1e-15
