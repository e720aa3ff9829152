"""Seeded synthetic inputs for the loss pass (test and benchmark harness, not part of the path).

The five workloads mirror the shapes of buffered rollouts in short-horizon reasoning, multi-turn
tool use and long-horizon coding-agent training at Qwen-scale vocabulary; they stand in for the
paper's rollout data, which is not available.  This module does none of the method's
arithmetic on behalf of the library or of the oracle: both receive the arrays made here.  The
only model-like step is drawing the sampled token and its reference log-probability with the
tensor library's own ``log_softmax`` so that the stored log-probabilities are realistic.

Everything is a function of (name, seed, overrides) and of the device's random generator, so
the same call gives the same arrays on the same device type.
"""

import numpy as np
import torch

CONFIGS = {
    # B samples of fixed length, all trainable
    "tiny": dict(V=4096, dtype="f32", B=4, len_lo=128, len_hi=128, structure="plain",
                 logit="normal", sigma=2.0, boost=0, lags=[0, 1, 2, 3], behav_sigma=0.05,
                 teacher_mu=-0.3, teacher_sigma=0.5, stale_sigma=0.0),
    "reasoning": dict(V=151936, dtype="bf16", B=64, len_lo=512, len_hi=4096, structure="plain",
                      logit="normal", sigma=3.0, boost=32, lag_lo=0, lag_hi=4, behav_sigma=0.05,
                      teacher_mu=-0.2, teacher_sigma=0.4, stale_sigma=0.0),
    # 8 turns: masked observation span then trainable response span
    "tooluse": dict(V=151936, dtype="bf16", B=32, structure="turns", turns=8, resp_lo=256, resp_hi=1024,
                    obs_lo=128, obs_hi=512, logit="normal", sigma=3.0, boost=32, lag_lo=0, lag_hi=8,
                    behav_sigma=0.05, teacher_mu=-0.2, teacher_sigma=0.4, stale_sigma=0.0),
    # fixed total length, alternating trainable / masked spans, stale teacher context present
    "coding": dict(V=151936, dtype="bf16", B=8, structure="spans", total_len=32768, resp_lo=512, resp_hi=2048,
                   obs_lo=256, obs_hi=1536, logit="normal", sigma=3.0, boost=32, lag_lo=0, lag_hi=16,
                   behav_sigma=0.05, teacher_mu=-0.2, teacher_sigma=0.4, stale_sigma=0.1, chunk=16384),
    "largevocab": dict(V=262144, dtype="bf16", B=16, len_lo=16384, len_hi=16384, structure="plain",
                       logit="student_t3", sigma=2.0, boost=0, lag_split=(8, 32), behav_sigma=0.05,
                       teacher_mu=-0.2, teacher_sigma=0.4, stale_sigma=0.0),
}


def _structure(cfg, rs):
    """seq_lens [B], mask [T] (numpy) for the workload's turn structure."""
    B = cfg["B"]
    lens, masks = [], []
    for _ in range(B):
        if cfg["structure"] == "plain":
            n = int(rs.randint(cfg["len_lo"], cfg["len_hi"] + 1))
            m = np.ones(n, dtype=np.uint8)
        elif cfg["structure"] == "turns":
            parts = []
            for _ in range(cfg["turns"]):
                parts.append(np.zeros(int(rs.randint(cfg["obs_lo"], cfg["obs_hi"] + 1)), dtype=np.uint8))
                parts.append(np.ones(int(rs.randint(cfg["resp_lo"], cfg["resp_hi"] + 1)), dtype=np.uint8))
            m = np.concatenate(parts)
        elif cfg["structure"] == "spans":
            total = cfg["total_len"]
            parts, have, train = [], 0, True
            while have < total:
                lo, hi = (cfg["resp_lo"], cfg["resp_hi"]) if train else (cfg["obs_lo"], cfg["obs_hi"])
                n = min(int(rs.randint(lo, hi + 1)), total - have)
                parts.append(np.full(n, 1 if train else 0, dtype=np.uint8))
                have += n
                train = not train
            m = np.concatenate(parts)
        else:
            raise ValueError(cfg["structure"])
        lens.append(len(m))
        masks.append(m)
    return np.array(lens, dtype=np.int32), np.concatenate(masks)


def _lags(cfg, rs):
    B = cfg["B"]
    if "lags" in cfg:
        return np.array([cfg["lags"][i % len(cfg["lags"])] for i in range(B)], dtype=np.int32)
    if "lag_split" in cfg:                       # first half fresh, second half very stale
        lo, hi = cfg["lag_split"]
        lag = np.zeros(B, dtype=np.int32)
        lag[B // 2:] = rs.randint(lo, hi + 1, size=B - B // 2)
        return lag
    return rs.randint(cfg["lag_lo"], cfg["lag_hi"] + 1, size=B).astype(np.int32)


def _logit_rows(cfg, rows, V, gen, device):
    """[rows, V] float32 raw logits before rounding to the storage type."""
    if cfg["logit"] == "normal":
        z = torch.randn(rows, V, generator=gen, device=device) * cfg["sigma"]
    elif cfg["logit"] == "student_t3":           # heavy tails: t with 3 degrees of freedom
        z = torch.randn(rows, V, generator=gen, device=device)
        chi = torch.zeros(rows, V, device=device)
        for _ in range(3):
            chi += torch.randn(rows, V, generator=gen, device=device) ** 2
        z = z * torch.rsqrt(chi / 3.0) * cfg["sigma"]
        del chi
    else:
        raise ValueError(cfg["logit"])
    if cfg["boost"] > 0:                         # a few strongly preferred tokens per row
        idx = torch.randint(0, V, (rows, cfg["boost"]), generator=gen, device=device)
        z.scatter_(1, idx, z.gather(1, idx) + 8.0)
    return z


def generate(name, device="cpu", seed=0, row_block=1024, ld=None, **overrides):
    """Builds one workload.  Returns a dict of tensors on `device` plus plain metadata.

    overrides replace entries of CONFIGS[name] (e.g. B=8, V=4096, len_hi=600) to make the
    reduced-size replicas the tests use.  aligned_split=(a, b) turns a fraction a of the kept rows into
    "rollout-aligned only" (mask 2) and a fraction b into "supervision-aligned only" (mask 3), so that the
    two aligned sets of a sample differ.  stale_logit_sigma=s (> 0) also returns `logits_stale`:
    the logits a stale checkpoint would give on the same prefixes, logits + s * lag_i * N(0, 1)
    per entry (identical to the current ones for lag 0), for the full-vocabulary drift diagnostic.
    teacher_list=(k, s) also returns `list_ids` [T, k] int32 and `list_logp` [T, k] f32: the k most likely tokens
    of a teacher whose logits are logits + s * N(0, 1) per entry, and their log-probabilities (the tensor library's
    top-k and log-softmax: input preparation), from a generator of their own so that the other arrays do not change.
    """
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    V = int(cfg["V"])
    ld = V if ld is None else int(ld)
    dtype = torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16
    rs = np.random.RandomState(seed)
    seq_lens, mask = _structure(cfg, rs)
    lag = _lags(cfg, rs)
    if "aligned_split" in cfg:
        a, b = cfg["aligned_split"]
        u = np.random.RandomState(seed + 7919).uniform(size=mask.shape[0])
        mask = np.where((mask != 0) & (u < a), 2, np.where((mask != 0) & (u < a + b), 3, mask)).astype(np.uint8)
    T = int(seq_lens.sum())
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed * 1000003 + 17)

    logits = torch.empty(T, ld, dtype=dtype, device=dev)
    if ld > V:
        logits[:, V:] = 0
    stale_sigma = float(cfg.get("stale_logit_sigma", 0.0))
    logits_stale = torch.zeros(T, ld, dtype=dtype, device=dev) if stale_sigma > 0 else None
    lag_rows = torch.from_numpy(np.repeat(lag, seq_lens).astype(np.float32)).to(dev)
    token_ids = torch.empty(T, dtype=torch.int32, device=dev)
    ref_logp = torch.empty(T, dtype=torch.float32, device=dev)
    list_ids = list_logp = None
    if "teacher_list" in cfg:
        list_k, list_sigma = int(cfg["teacher_list"][0]), float(cfg["teacher_list"][1])
        list_ids = torch.empty(T, list_k, dtype=torch.int32, device=dev)
        list_logp = torch.empty(T, list_k, dtype=torch.float32, device=dev)
        gen_list = torch.Generator(device=dev)
        gen_list.manual_seed(seed * 1000003 + 31)
    for a in range(0, T, row_block):
        b = min(a + row_block, T)
        zraw = _logit_rows(cfg, b - a, V, gen, dev)
        z = zraw.to(dtype)
        logits[a:b, :V] = z
        if list_ids is not None:
            zq = z.float() + list_sigma * torch.randn(b - a, V, generator=gen_list, device=dev)
            top = torch.topk(zq, list_k, dim=1)
            list_ids[a:b] = top.indices.to(torch.int32)
            list_logp[a:b] = top.values - torch.logsumexp(zq, dim=1, keepdim=True)
            del zq, top
        if logits_stale is not None:
            drift = torch.randn(b - a, V, generator=gen, device=dev) * (stale_sigma * lag_rows[a:b, None])
            logits_stale[a:b, :V] = torch.where(lag_rows[a:b, None] > 0, (zraw + drift).to(dtype), z)
            del drift
        del zraw
        zf = z.float()
        u = torch.rand(b - a, V, generator=gen, device=dev).clamp_(1e-20, 1.0)
        y = torch.argmax(zf - torch.log(-torch.log(u)), dim=1)      # Gumbel-max draw from softmax(z)
        token_ids[a:b] = y.to(torch.int32)
        ref_logp[a:b] = torch.log_softmax(zf, dim=1).gather(1, y[:, None])[:, 0]
        del z, zf, u, y

    per_tok_lag = torch.from_numpy(np.repeat(lag, seq_lens).astype(np.float32)).to(dev)
    n1 = torch.randn(T, generator=gen, device=dev)
    n2 = torch.randn(T, generator=gen, device=dev)
    n3 = torch.randn(T, generator=gen, device=dev)
    behav = torch.clamp(ref_logp + cfg["behav_sigma"] * per_tok_lag * n1, max=0.0)
    teacher = torch.clamp(ref_logp + cfg["teacher_mu"] + cfg["teacher_sigma"] * n2, max=0.0)
    stale = None
    if cfg["stale_sigma"] > 0:
        stale = torch.clamp(teacher + cfg["stale_sigma"] * per_tok_lag * n3, max=0.0)

    return dict(name=name, cfg=cfg, T=T, V=V, ld=ld, B=int(cfg["B"]), dtype=cfg["dtype"],
                logits=logits, logits_stale=logits_stale, token_ids=token_ids, mask=torch.from_numpy(mask).to(dev),
                behav_logp=behav, teacher_logp=teacher, teacher_logp_stale=stale, list_ids=list_ids,
                list_logp=list_logp,
                seq_lens=torch.from_numpy(seq_lens).to(dev), lag=torch.from_numpy(lag).to(dev),
                seq_lens_host=seq_lens, lag_host=lag, mask_host=mask,
                n_trainable=int(((mask != 0) & (mask != 2)).sum()))


def structure_only(name, seed=0, **overrides):
    """seq_lens [B] and mask [T] (numpy) that generate(name, seed=seed) would use, without any tensor."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    return _structure(cfg, np.random.RandomState(seed))


def generate_lm_head(T, d, V, device="cpu", seed=0, logit_sigma=3.0, masked_every=0, row_block=2048, ldh=None,
                     ldw=None):
    """Hidden states and an output projection whose logits have the spread of the stored-logits
    workloads: hidden ~ N(0, 1), weight ~ N(0, (logit_sigma / sqrt(d))^2), both bf16.  Token ids are drawn
    from softmax of the projected row (Gumbel-max, in row blocks, with the tensor library's matmul: this
    is input preparation, not part of the path).  masked_every = m > 0 masks every m-th row."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed * 1000003 + 29)
    ldh = d if ldh is None else int(ldh)
    ldw = d if ldw is None else int(ldw)
    hidden = torch.zeros(T, ldh, dtype=torch.bfloat16, device=dev)
    weight = torch.zeros(V, ldw, dtype=torch.bfloat16, device=dev)
    for a in range(0, T, 8192):
        b = min(a + 8192, T)
        hidden[a:b, :d] = torch.randn(b - a, d, generator=gen, device=dev).to(torch.bfloat16)
    for a in range(0, V, 8192):
        b = min(a + 8192, V)
        weight[a:b, :d] = (torch.randn(b - a, d, generator=gen, device=dev) * (logit_sigma / d ** 0.5)).to(torch.bfloat16)
    token_ids = torch.empty(T, dtype=torch.int32, device=dev)
    wt = weight[:, :d].float().t().contiguous() if dev.type == "cpu" else None
    for a in range(0, T, row_block):
        b = min(a + row_block, T)
        if wt is not None:
            z = hidden[a:b, :d].float() @ wt
        else:
            z = (hidden[a:b, :d] @ weight[:, :d].t()).float()
        u = torch.rand(b - a, V, generator=gen, device=dev).clamp_(1e-20, 1.0)
        token_ids[a:b] = torch.argmax(z - torch.log(-torch.log(u)), dim=1).to(torch.int32)
        del z, u
    mask = torch.ones(T, dtype=torch.uint8, device=dev)
    if masked_every > 0:
        mask[::masked_every] = 0
    return dict(T=T, d=d, V=V, ldh=ldh, ldw=ldw, hidden=hidden, weight=weight, token_ids=token_ids, mask=mask)


def attach_loss_inputs(h, seq_lens, lag, seed=0, behav_sigma=0.05, teacher_mu=-0.2, teacher_sigma=0.4, row_block=2048,
                       teacher_list=None):
    """Adds to a generate_lm_head() dict what the loss pass needs besides hidden states and the projection:
    seq_lens / lag (given, numpy int32; sum(seq_lens) == T) and the stored log-probabilities
    behav_logp = min(lp + behav_sigma * lag_i * N(0,1), 0), teacher_logp = min(lp + N(teacher_mu, teacher_sigma^2), 0),
    where lp is the tensor library's log_softmax of the projected row at the drawn token (input preparation).
    teacher_list=(k, s) also adds `list_ids`, `list_logp` [T, k]: the k most likely tokens of a teacher whose logits
    are the projected row + s * N(0, 1) per entry, and their log-probabilities."""
    dev = h["hidden"].device
    T, d, V = h["T"], h["d"], h["V"]
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    lag = np.asarray(lag, dtype=np.int32)
    assert int(seq_lens.sum()) == T and len(lag) == len(seq_lens)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed * 1000003 + 41)
    ref = torch.empty(T, dtype=torch.float32, device=dev)
    list_ids = list_logp = None
    if teacher_list is not None:
        list_ids = torch.empty(T, int(teacher_list[0]), dtype=torch.int32, device=dev)
        list_logp = torch.empty(T, int(teacher_list[0]), dtype=torch.float32, device=dev)
        gen_list = torch.Generator(device=dev)
        gen_list.manual_seed(seed * 1000003 + 43)
    wt = h["weight"][:, :d].float().t().contiguous() if dev.type == "cpu" else None
    for a in range(0, T, row_block):
        b = min(a + row_block, T)
        if wt is not None:
            z = h["hidden"][a:b, :d].float() @ wt
        else:
            z = (h["hidden"][a:b, :d] @ h["weight"][:, :d].t()).float()
        ref[a:b] = torch.log_softmax(z, dim=1).gather(1, h["token_ids"][a:b].long()[:, None])[:, 0]
        if teacher_list is not None:
            zq = z + float(teacher_list[1]) * torch.randn(b - a, V, generator=gen_list, device=dev)
            top = torch.topk(zq, int(teacher_list[0]), dim=1)
            list_ids[a:b] = top.indices.to(torch.int32)
            list_logp[a:b] = top.values - torch.logsumexp(zq, dim=1, keepdim=True)
            del zq, top
        del z
    per_tok_lag = torch.from_numpy(np.repeat(lag, seq_lens).astype(np.float32)).to(dev)
    n1 = torch.randn(T, generator=gen, device=dev)
    n2 = torch.randn(T, generator=gen, device=dev)
    out = dict(h)
    out.update(B=len(seq_lens), seq_lens=torch.from_numpy(seq_lens).to(dev), lag=torch.from_numpy(lag).to(dev),
               seq_lens_host=seq_lens, lag_host=lag,
               behav_logp=torch.clamp(ref + behav_sigma * per_tok_lag * n1, max=0.0),
               teacher_logp=torch.clamp(ref + teacher_mu + teacher_sigma * n2, max=0.0), list_ids=list_ids,
               list_logp=list_logp)
    return out
