"""The pins must fail when the oracle is wrong.  Each case plants one plausible mistake (a dropped term, a
wrong sign, a swapped operand, a wrong normaliser) in a copy of the oracle's source, loads that copy as a
module and runs the pin tests with it in place of the real oracle; at least one pin has to fail.  CPU
only: the mistakes live in the oracle, never in the GPU path."""

import os
import types

import pytest

import test_oracle_pins as pins
import test_refresh_rule as refresh_pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_SRC = open(os.path.join(ROOT, "oracle", "fopd_oracle.py")).read()

MISTAKES = {
    "advantage sign": ("adv = lq - lp                        # OPD advantage against the teacher",
                       "adv = lp - lq"),
    "drift estimator loses its -rho + 1": ("k_roll = rho * delta - rho + 1.0", "k_roll = rho * delta"),
    "estimator of the opposite KL direction": ("return r * d - r + 1.0", "return r - 1.0 - d"),
    "lag enters as tau instead of tau + 1": ("f[i] = math.exp(-surrogate) / (int(lag[i]) + 1)",
                                             "f[i] = math.exp(-surrogate) / max(int(lag[i]), 1)"),
    "alpha and beta swapped": ("surrogate = alpha * math.sqrt(D_roll[i]) + beta * math.sqrt(D_sup[i])",
                               "surrogate = beta * math.sqrt(D_roll[i]) + alpha * math.sqrt(D_sup[i])"),
    "square roots dropped": ("surrogate = alpha * math.sqrt(D_roll[i]) + beta * math.sqrt(D_sup[i])",
                             "surrogate = alpha * D_roll[i] + beta * D_sup[i]"),
    "gate keeps f instead of f - xi": ("w[i] = max(float(f[i]) - xi, 0.0)",
                                       "w[i] = float(f[i]) if float(f[i]) > xi else 0.0"),
    "loss normalised by surviving samples": (
        "return math.fsum(float(w[i]) * (float(ell[i]) + lam * float(D_roll[i])) for i in range(B)) / B",
        "return math.fsum(float(w[i]) * (float(ell[i]) + lam * float(D_roll[i])) for i in range(B)) / "
        "max(1, sum(1 for i in range(B) if w[i] > 0))"),
    "anchor gradient sign": ("part -= lam * rho[t] * delta[t] / int(n_roll[i])",
                             "part += lam * rho[t] * delta[t] / int(n_roll[i])"),
    "anchor gradient loses rho": ("part -= lam * rho[t] * delta[t] / int(n_roll[i])",
                                  "part -= lam * delta[t] / int(n_roll[i])"),
    "coefficient normalised by H instead of n": (
        "part += adv[t] / int(n_train[i])", "part += adv[t] / int(cu[i + 1] - cu[i])"),
    "anchor normalised by the supervision count": ("part -= lam * rho[t] * delta[t] / int(n_roll[i])",
                                                   "part -= lam * rho[t] * delta[t] / int(n_train[i])"),
    "rollout drift averaged over the supervision set": (
        "D_roll[i] = math.fsum(float(k_roll[t]) for t in rows_roll) / int(n_roll[i])",
        "D_roll[i] = math.fsum(float(k_roll[t]) for t in rows) / int(n[i])"),
    "token loss averaged over the rollout set": (
        "            ell[i] = math.fsum(float(lp[t] - lq[t]) for t in rows) / int(n[i])",
        "            ell[i] = math.fsum(float(lp[t] - lq[t]) for t in rows_roll) / int(n_roll[i])"),
    "sample stays valid with one aligned set empty": (
        "        if n[i] == 0 or n_roll[i] == 0:\n            continue\n        rows = ",
        "        if n[i] == 0 and n_roll[i] == 0:\n            continue\n        rows = "),
    "weights ignore an empty rollout set": ("    w = freshness_weights(f, xi, n_valid)\n    loss = anchored_loss(w, ell, D_roll, lam)\n    coef",
                                            "    w = freshness_weights(f, xi, n)\n    loss = anchored_loss(w, ell, D_roll, lam)\n    coef"),
    "roll coverage reported as sup coverage": (
        "mroll = mbar if cover_roll is None else math.fsum(float(x) for x in cover_roll) / B", "mroll = mbar"),
    "aligned sets swapped": ("    return int(m) != 0 and int(m) != 2\n", "    return int(m) != 0 and int(m) != 3\n"),
    "unit rows keep the sample weight": (
        "coef_unit = grad_coefficients(delta, rho, adv, mask, cu, n, ones, lam, grad_scale, n_roll=n_roll)",
        "coef_unit = grad_coefficients(delta, rho, adv, mask, cu, n, w, lam, grad_scale, n_roll=n_roll)"),
    "unit rows lose the upstream scale": (
        "coef_unit = grad_coefficients(delta, rho, adv, mask, cu, n, ones, lam, grad_scale, n_roll=n_roll)",
        "coef_unit = grad_coefficients(delta, rho, adv, mask, cu, n, ones, lam, 1.0, n_roll=n_roll)"),
    "listed-token teacher: the rest event dropped": (
        "        ell += p_rest * g_rest\n        G[~in_list] = g_rest", "        G[~in_list] = g_rest"),
    "listed-token teacher: forward instead of reverse KL": (
        "        G[u] = logp[u] - float(logq[j])\n        if p[u] > 0.0:\n            ell += p[u] * G[u]",
        "        G[u] = logp[u] - float(logq[j])\n        if p[u] > 0.0:\n            ell -= math.exp(float(logq[j])) * G[u]"),
    "listed-token teacher: rest of the teacher not floored": (
        "q_rest = max(1.0 - q_listed, float(rest_floor))", "q_rest = max(1.0 - q_listed, 1e-300)"),
    "listed-token teacher: rest of the student taken as one token": (
        "p_rest = float(np.sum(p[~in_list]))", "p_rest = float(np.max(p[~in_list])) if np.any(~in_list) else 0.0"),
    "listed-token teacher: gradient not centred by the loss": (
        "g = p * (c1_t + c2_t * (np.where(p > 0.0, G, 0.0) - ell))", "g = p * (c1_t + c2_t * np.where(p > 0.0, G, 0.0))"),
    "listed-token teacher: token loss normalised by the rollout count": (
        "            if in_sup_set(mask[t]):\n                c2[t] = grad_scale * w[i] / (B * int(n[i]))\n    res = dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, lse=lse, logp=lp, token_loss=tok",
        "            if in_sup_set(mask[t]):\n                c2[t] = grad_scale * w[i] / (B * int(n_roll[i]))\n    res = dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, lse=lse, logp=lp, token_loss=tok"),
    "listed-token teacher: supervision drift kept without the stale array": (
        "    if teacher_logp is None or teacher_logp_stale is None:\n        k_sup = np.zeros(T)",
        "    if teacher_logp is None:\n        k_sup = np.zeros(T)\n    elif teacher_logp_stale is None:\n        k_sup = kl_estimator(np.asarray(teacher_logp, dtype=np.float64))"),
    "listed-token teacher through the projection: rows contracted unrounded": (
        'g, gb = res["dlogits_exact"], res["dlogits"]', 'g, gb = res["dlogits_exact"], res["dlogits_exact"]'),
    "listed-token teacher through the projection: weight gradient contracts over the wrong axis": (
        "               dhidden_exact=np.matmul(g, weight), dweight_exact=np.matmul(g.T, hidden))",
        "               dhidden_exact=np.matmul(g, weight), dweight_exact=np.matmul(g.T, hidden)[::-1])"),
    "one-hot not subtracted": ("    g[y] -= 1.0\n    return c_t * g", "    return c_t * g"),
    "log-sum-exp forgets the shift": ("return float(mx + np.log(np.sum(np.exp(z - mx))))",
                                      "return float(np.log(np.sum(np.exp(z - mx))))"),
    "token means over all rows": ("ell[i] = math.fsum(float(lp[t] - lq[t]) for t in rows) / int(n[i])",
                                  "ell[i] = math.fsum(float(lp[t] - lq[t]) for t in rows) / H"),
    "coverage inverted": ("cover[i] = int(n[i]) / H", "cover[i] = H / max(int(n[i]), 1)"),
    "bf16 rounding truncates": ("r = np.rint(x[fin] / quantum) * quantum", "r = np.trunc(x[fin] / quantum) * quantum"),
    "mask ignored in the counts": ("            if in_sup_set(mask[t]):\n                cnt += 1", "            cnt += 1"),
    "offsets start at the first length": ("cu[i + 1] = cu[i] + int(seq_lens[i])",
                                          "cu[i + 1] = cu[i] + int(seq_lens[min(i + 1, seq_lens.shape[0] - 1)])"),
    "gather index with the wrong pitch": ("out[t] = int(t) * int(ld) + int(token_ids[t])",
                                          "out[t] = int(t) * (int(ld) - 1) + int(token_ids[t])"),
    "full KL weighted by the stale distribution": (
        "kl[t] = float(np.sum(np.where(p > 0.0, p * (np.where(p > 0.0, logp, 0.0) - logq), 0.0)))",
        "kl[t] = float(np.sum(np.exp(logq) * (logp - logq)))"),
    "full-KL gradient forgets the -KL centring": ("g = p * (c1_t + c2_t * ((logp - (zs - lse_stale_t)) - kl_t))",
                                                  "g = p * (c1_t + c2_t * (logp - (zs - lse_stale_t)))"),
    "entropy sign": ("H[t] = -float(np.sum(", "H[t] = float(np.sum("),
    "refresh uses < for mean freshness": ("if fbar <= kappa_f:", "if fbar < kappa_f:"),
    "refresh rate limit off by one": ("step - last_refresh_step >= min_interval", "step - last_refresh_step > min_interval"),
    "invalid samples keep a weight": ("        if int(n_train[i]) == 0:\n            continue\n        w[i] = max(",
                                      "        w[i] = max("),
    "ratio linearised": ("rho = np.exp(delta)                  # importance ratio, not clipped", "rho = 1.0 + delta"),
    "supervision drift averages the rollout terms": (
        "D_sup[i] = math.fsum(float(k_sup[t]) for t in rows) / int(n[i])",
        "D_sup[i] = math.fsum(float(k_roll[t]) for t in rows) / int(n[i])"),
    "buffer means over valid samples only": ("fbar = math.fsum(float(x) for x in f) / B",
                                             "fbar = math.fsum(float(x) for x in f) / max(1, sum(1 for x in f if x > 0))"),
    "upstream scale dropped": ("c[t] = grad_scale * w[i] / B * part", "c[t] = w[i] / B * part"),
    "bf16 spacing one bit too fine": ("quantum = np.ldexp(1.0, e - 7)          # spacing of bf16 numbers in that binade",
                                      "quantum = np.ldexp(1.0, e - 8)"),
    "full-teacher anchor sign": ("c1[t] = -grad_scale * w[i] / (B * int(n_roll[i])) * lam * rho[t] * delta[t]",
                                 "c1[t] = grad_scale * w[i] / (B * int(n_roll[i])) * lam * rho[t] * delta[t]"),
    "full-KL variant drops the advantage": ("c1[t] = grad_scale * w[i] / (B * int(n[i])) * adv[t]", "c1[t] = 0.0"),
    "full-KL anchor over the supervision set": ("c2[t] = grad_scale * w[i] / (B * int(n_roll[i])) * lam",
                                                "c2[t] = grad_scale * w[i] / (B * int(n[i])) * lam"),
    "projection contracts the wrong axis": ("return np.matmul(hidden, weight.T)",
                                            "return np.matmul(hidden, weight[:, ::-1].T)"),
    "projection returns vocabulary-major logits": ("return np.matmul(hidden, weight.T)",
                                                   "return np.matmul(weight, hidden.T)"),
    "supervision drift averaged over the rollout set": (
        "D_sup[i] = math.fsum(float(k_sup[t]) for t in rows) / int(n[i])",
        "D_sup[i] = math.fsum(float(k_sup[t]) for t in rows_roll) / int(n_roll[i])"),
    "roll coverage counts the supervision set": (
        "cover_roll[i] = int(n_roll[i]) / (int(cu[i + 1]) - int(cu[i]))",
        "cover_roll[i] = int(n[i]) / (int(cu[i + 1]) - int(cu[i]))"),
    "validity looks at the supervision set only": ("return cover_roll, n_roll, np.minimum(n, n_roll)",
                                                   "return cover_roll, n_roll, n"),
    "projection gradient: hidden-state gradient contracts the wrong axis": (
        "dhidden_exact=np.matmul(g, weight), dweight_exact=np.matmul(g.T, hidden))",
        "dhidden_exact=np.matmul(g, weight[::-1]), dweight_exact=np.matmul(g.T, hidden))"),
    "projection gradient: weight gradient pairs rows with the wrong tokens": (
        "dhidden_exact=np.matmul(g, weight), dweight_exact=np.matmul(g.T, hidden))",
        "dhidden_exact=np.matmul(g, weight), dweight_exact=np.matmul(g.T, hidden[::-1]))"),
    "projection gradient: rows not rounded to the storage type before the contractions": (
        "    gb = round_to_bf16(g)\n    return dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, logits=z,",
        "    gb = g\n    return dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, logits=z,"),
    "projection gradient: supplied scores ignored": (
        "    w = freshness_weights(np.asarray(freshness, dtype=np.float64), xi, n_valid)\n    loss = anchored_loss(w, ell, D_roll, lam)\n    coef = grad_coefficients(delta, rho, adv, mask, cu, n, w, lam, grad_scale, n_roll=n_roll)\n    g = np.zeros((T, V))",
        "    w = freshness_weights(np.ones(len(n)), xi, n_valid)\n    loss = anchored_loss(w, ell, D_roll, lam)\n    coef = grad_coefficients(delta, rho, adv, mask, cu, n, w, lam, grad_scale, n_roll=n_roll)\n    g = np.zeros((T, V))"),
    "stale teacher difference reversed": ("eps = lq - np.asarray(teacher_logp_stale, dtype=np.float64)",
                                          "eps = np.asarray(teacher_logp_stale, dtype=np.float64) - lq"),
}


def _load(source):
    mod = types.ModuleType("fopd_oracle_under_test")
    exec(compile(source, "fopd_oracle_under_test.py", "exec"), mod.__dict__)
    return mod


def _pin_calls():
    """Every pin test as a (name, zero-argument callable), parametrised ones expanded."""
    calls = []
    for module in (pins, refresh_pins):
        for name, fn in sorted(vars(module).items()):
            if not name.startswith("test_") or not callable(fn):
                continue
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if not marks:
                calls.append((name, fn))
                continue
            argnames = [a.strip() for a in marks[0].args[0].split(",")]
            for values in marks[0].args[1]:
                values = values if isinstance(values, (tuple, list)) else (values,)
                calls.append(("%s%s" % (name, list(values)), (lambda f=fn, kw=dict(zip(argnames, values)): f(**kw))))
    return calls


def _first_failing_pin(oracle_module, skip=()):
    saved = pins.orc, refresh_pins.orc
    pins.orc = refresh_pins.orc = oracle_module
    try:
        for name, call in _pin_calls():
            if any(name.startswith(s) for s in skip):
                continue
            try:
                call()
            except Exception:          # an assertion, or the broken oracle raising on its own
                return name
        return None
    finally:
        pins.orc, refresh_pins.orc = saved


def test_control_an_unchanged_copy_passes():
    assert len(_pin_calls()) >= 30
    assert _first_failing_pin(_load(ORACLE_SRC)) is None


@pytest.mark.parametrize("name", sorted(MISTAKES))
def test_planted_mistake_is_caught(name):
    old, new = MISTAKES[name]
    assert ORACLE_SRC.count(old) >= 1, "the oracle no longer contains: " + old
    caught_by = _first_failing_pin(_load(ORACLE_SRC.replace(old, new)))
    assert caught_by is not None, "no pin noticed: " + name


# The two tests that compare the oracle with a second typing of the same formulas share an author with it and
# can share a misreading, so they do not count as pins for what the paper fixes by definition: with both set
# aside, the mistakes below (each contradicting Eq. "sample-aggregated-loss", Eq. "kl-diagnostics" line 2,
# the aggregates of Sec. 4.2 or Algorithm 1's invalid-sample branch) must still be caught - by the hand-worked
# fixture, closed forms, enumeration or finite differences.
REIMPLEMENTATIONS = ("test_whole_pass_matches_scalar_reimplementation",
                     "test_two_aligned_sets_against_scalar_reimplementation")
FIXED_BY_DEFINITION = ["token means over all rows", "token loss averaged over the rollout set",
                       "supervision drift averages the rollout terms", "roll coverage reported as sup coverage",
                       "weights ignore an empty rollout set", "rollout drift averaged over the supervision set",
                       "sample stays valid with one aligned set empty", "aligned sets swapped",
                       "anchor normalised by the supervision count", "coefficient normalised by H instead of n",
                       "loss normalised by surviving samples", "buffer means over valid samples only",
                       "coverage inverted", "invalid samples keep a weight",
                       "supervision drift averaged over the rollout set", "roll coverage counts the supervision set",
                       "validity looks at the supervision set only"]


@pytest.mark.parametrize("name", FIXED_BY_DEFINITION)
def test_caught_without_the_reimplementation_tests(name):
    old, new = MISTAKES[name]
    caught_by = _first_failing_pin(_load(ORACLE_SRC.replace(old, new)), skip=REIMPLEMENTATIONS)
    assert caught_by is not None, "only a re-typed formula noticed: " + name


def test_every_mistake_is_caught_without_the_reimplementation_tests():
    missed = [name for name, (old, new) in sorted(MISTAKES.items())
              if _first_failing_pin(_load(ORACLE_SRC.replace(old, new)), skip=REIMPLEMENTATIONS) is None]
    assert missed == [], missed
