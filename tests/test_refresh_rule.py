"""Adaptive refresh test: the host-side C function against the oracle and against the inequalities
written out from Sec. 4.2 (mean freshness uses <=, the two coverage means use <) and the rate limit of
App. B (at most one refresh per min_interval optimizer steps).  CPU only."""

import itertools

import numpy as np

from oracle import fopd_oracle as orc
from paper_2605_17862_amd import binding as fb


def test_truth_table_of_the_three_conditions():
    cfg = fb.RefreshConfig(0.3, 0.5, 0.6, 1)
    cases = {
        (0.31, 0.5, 0.6): 0,          # all at or above their thresholds: coverage equal is still fine
        (0.30, 0.5, 0.6): 1,          # mean freshness equal to kappa_f refreshes (<=)
        (0.29, 0.9, 0.9): 1,
        (0.9, 0.4999, 0.9): 2,
        (0.9, 0.9, 0.5999): 4,
        (0.1, 0.1, 0.1): 7,
        (0.9, 0.5, 0.61): 0,
    }
    for step, (agg, want) in enumerate(cases.items()):
        state = fb.RefreshState()
        got, reason = fb.fopd_refresh_decide(agg, cfg, state, step)
        assert reason == want and got == (want != 0), (agg, reason, got)
        ref, reasons = orc.refresh_decision(np.float32(agg), np.float32(0.3), np.float32(0.5), np.float32(0.6),
                                            step, None, 1)
        assert ref == got and reason == sum({"f": 1, "roll": 2, "sup": 4}[r] for r in reasons)
        assert state.refreshes == int(got) and state.last_refresh_step == (step if got else -1)


def test_rate_limit_of_one_refresh_per_interval():
    cfg = fb.RefreshConfig(0.5, 0.0, 0.0, 200)
    state = fb.RefreshState()
    stale = (0.1, 1.0, 1.0)
    fired = [t for t in range(0, 1000) if fb.fopd_refresh_decide(stale, cfg, state, t)[0]]
    assert fired == [0, 200, 400, 600, 800] and state.refreshes == 5
    # a fresh buffer never refreshes, and does not reset the clock
    state = fb.RefreshState()
    assert not fb.fopd_refresh_decide((0.9, 1.0, 1.0), cfg, state, 5)[0] and state.last_refresh_step == -1
    assert fb.fopd_refresh_decide(stale, cfg, state, 7) == (True, 1)
    assert fb.fopd_refresh_decide(stale, cfg, state, 206) == (False, 1)       # reason reported, refresh held back
    assert fb.fopd_refresh_decide(stale, cfg, state, 207) == (True, 1)


def test_random_sequences_against_oracle():
    rng = np.random.default_rng(3)
    for interval, trial in itertools.product((1, 3, 10), range(5)):
        cfg = fb.RefreshConfig(0.4, 0.5, 0.5, interval)
        state = fb.RefreshState()
        last = None
        for step in range(60):
            agg = rng.uniform(0.2, 0.8, size=3).astype(np.float32)
            got, _ = fb.fopd_refresh_decide(agg, cfg, state, step)
            want, _ = orc.refresh_decision(agg, np.float32(0.4), np.float32(0.5), np.float32(0.5), step, last, interval)
            assert got == want
            if want:
                last = step
        assert state.last_refresh_step == (-1 if last is None else last)


def test_bad_arguments():
    lib = fb.load_library()
    cfg = fb.RefreshConfig(0.4, 0.5, 0.5, 0)
    state = fb.RefreshState()
    import ctypes
    arr = (ctypes.c_float * 3)(0.1, 0.1, 0.1)
    assert lib.fopd_refresh_decide(arr, ctypes.byref(cfg), ctypes.byref(state), 0, None) == -1
    cfg.min_interval = 1
    assert lib.fopd_refresh_decide(None, ctypes.byref(cfg), ctypes.byref(state), 0, None) == -1
    assert lib.fopd_refresh_decide(arr, ctypes.byref(cfg), ctypes.byref(state), 0, None) == 1
