"""The synthetic input generator: determinism, structure and value ranges (CPU, reduced sizes)."""

import numpy as np
import torch

from harness import workloads as wl


def test_tiny_is_as_specified_and_deterministic():
    a = wl.generate("tiny", "cpu", seed=0)
    b = wl.generate("tiny", "cpu", seed=0)
    c = wl.generate("tiny", "cpu", seed=1)
    assert a["T"] == 512 and a["V"] == 4096 and a["B"] == 4 and a["logits"].dtype == torch.float32
    assert list(a["lag_host"]) == [0, 1, 2, 3] and a["n_trainable"] == 512
    assert torch.equal(a["logits"], b["logits"]) and torch.equal(a["token_ids"], b["token_ids"])
    assert torch.equal(a["behav_logp"], b["behav_logp"])
    assert not torch.equal(a["logits"], c["logits"])
    assert abs(float(a["logits"].std()) - 2.0) < 0.02
    assert float(a["teacher_logp"].max()) <= 0.0 and float(a["behav_logp"].max()) <= 0.0
    ref = torch.log_softmax(a["logits"].double(), 1).gather(1, a["token_ids"].long()[:, None])[:, 0]
    # lag 0 sample: stored behaviour log-prob is the reference log-prob itself
    assert torch.allclose(a["behav_logp"][:128].double(), ref[:128], atol=2e-6)
    assert float((a["behav_logp"][384:].double() - ref[384:]).std()) > 0.1
    assert a["token_ids"].min() >= 0 and a["token_ids"].max() < 4096


def test_turn_and_span_structures():
    w = wl.generate("tooluse", "cpu", seed=0, B=3, V=512)
    m = w["mask_host"]
    assert w["T"] == int(w["seq_lens_host"].sum()) == len(m)
    start = 0
    for n in w["seq_lens_host"]:
        seg = m[start:start + n]
        flips = int(np.sum(seg[1:] != seg[:-1]))
        assert seg[0] == 0 and seg[-1] == 1 and flips == 15      # 8 x (observation, response)
        start += n
    w = wl.generate("coding", "cpu", seed=0, B=2, V=512, total_len=8192)
    assert list(w["seq_lens_host"]) == [8192, 8192]
    frac = w["n_trainable"] / w["T"]
    assert 0.45 < frac < 0.75
    assert w["teacher_logp_stale"] is not None and w["logits"].dtype == torch.bfloat16


def test_boost_and_heavy_tails_and_padding():
    w = wl.generate("reasoning", "cpu", seed=0, B=2, len_lo=16, len_hi=24, V=4096, ld=4104)
    z = w["logits"][:, :4096].float()
    assert w["logits"].shape[1] == 4104 and float(w["logits"][:, 4096:].abs().max()) == 0.0
    assert float((z > 9.0).float().sum(1).mean()) > 8          # boosted ids stand out
    assert 0 <= int(w["lag_host"].min()) and int(w["lag_host"].max()) <= 4
    w = wl.generate("largevocab", "cpu", seed=0, B=4, len_lo=8, len_hi=8, V=8192)
    assert list(w["lag_host"][:2]) == [0, 0] and int(w["lag_host"][2:].min()) >= 8
    assert float(w["logits"].float().abs().max()) > 30.0        # Student-t tails


def test_aligned_split_marks_rows_and_leaves_the_rest_of_the_workload_alone():
    kw = dict(B=3, total_len=200, resp_lo=10, resp_hi=30, obs_lo=5, obs_hi=15, V=64)
    a = wl.generate("coding", "cpu", seed=4, **kw)
    b = wl.generate("coding", "cpu", seed=4, aligned_split=(0.3, 0.2), **kw)
    ma, mb = a["mask_host"], b["mask_host"]
    assert set(np.unique(ma)) <= {0, 1} and set(np.unique(mb)) == {0, 1, 2, 3}
    assert np.array_equal(ma != 0, mb != 0)                       # only kept rows are re-labelled
    kept = int((ma != 0).sum())
    assert abs(int((mb == 2).sum()) / kept - 0.3) < 0.08 and abs(int((mb == 3).sum()) / kept - 0.2) < 0.08
    assert b["n_trainable"] == int(((mb == 1) | (mb == 3)).sum())  # rows that carry the token loss
    assert np.array_equal(a["seq_lens_host"], b["seq_lens_host"]) and np.array_equal(a["lag_host"], b["lag_host"])
    assert bool((a["logits"] == b["logits"]).all()) and bool((a["token_ids"] == b["token_ids"]).all())
    c = wl.generate("coding", "cpu", seed=4, aligned_split=(0.3, 0.2), **kw)
    assert np.array_equal(mb, c["mask_host"])                      # seeded
