"""Benchmark of the fused f-OPD loss pass on one MI355X.

A step is one call of fopd_loss_fwd_bwd that does everything (token log-probs, drift diagnostics,
freshness scores, weights, loss, gradient) over the "reasoning" workload: B=64 ragged sequences,
V=151,936, bf16 logits, already resident in HBM.  Prints one JSON line.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PMC_SUMMARY = os.path.join(ROOT, "profiles", "fopd_loss_fwd_bwd_reasoning_pmc_hbm_traffic.txt")


def measured_traffic(workload, T, V, key):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE runs,
    scaled by the copy-kernel calibration), if that summary is for exactly this workload; else None."""
    try:
        kv = dict(l.strip().split(": ", 1) for l in open(PMC_SUMMARY) if ": " in l and not l.startswith(" "))
        if kv.get("workload") == workload and int(kv["T_rows"]) == T and int(kv["V"]) == V:
            return float(kv[key])
    except (OSError, KeyError, ValueError):
        pass
    return None


def _cpu_baseline_worker(job):
    """One whole sample through the oracle, as it stands.  Runs in a worker process (host only)."""
    import numpy as np
    from oracle import fopd_oracle as orc
    path, hp = job
    if path is None:                                   # warm-up task: imports only
        return 0
    d = np.load(path)
    z = (d["z16"].astype(np.uint32) << 16).view(np.float32).astype(np.float64)     # bf16 bits, widened exactly
    a, b, xi, lam = hp
    res = orc.fopd_loss_fwd_bwd(z, d["y"], d["m"], d["lb"], d["lq"], None, d["seq"], d["lag"], a, b, xi, lam,
                                out_dtype="bf16", want_dlogits=True)
    return int(res["n_train"].sum())


def cpu_baseline(w, hp, rows_per_core=1500):
    """The float64 oracle, as it stands, on whole samples of the same workload, one sample per task on a pool of
    worker processes over the host cores this process may use (at most 16, the share of a one-GPU machine)."""
    import multiprocessing as mp
    import shutil
    import tempfile
    from concurrent.futures import ProcessPoolExecutor
    import numpy as np
    from oracle import fopd_oracle as orc

    cores = max(1, min(len(os.sched_getaffinity(0)), 16))
    seq = w["seq_lens_host"]
    cu = orc.segment_offsets(seq)
    order = np.argsort(seq, kind="stable")
    chosen, rows = [], 0
    for i in order:
        chosen.append(int(i))
        rows += int(seq[i])
        if rows >= rows_per_core * cores and len(chosen) >= cores:
            break
    tmp = tempfile.mkdtemp(prefix="fopd_cpu_baseline_", dir="/dev/shm" if os.path.isdir("/dev/shm") else None)
    try:
        jobs = []
        for i in chosen:                                   # copies to the host are not timed
            s, e = int(cu[i]), int(cu[i + 1])
            path = os.path.join(tmp, "sample%d.npz" % i)
            zb = w["logits"][s:e, :w["V"]].contiguous()
            z16 = zb.view(__import__("torch").int16).cpu().numpy().view(np.uint16) if w["dtype"] == "bf16" else None
            if z16 is None:
                raise SystemExit("cpu_baseline: bf16 workloads only")
            np.savez(path, z16=z16, y=w["token_ids"][s:e].cpu().numpy(), m=w["mask_host"][s:e],
                     lb=w["behav_logp"][s:e].cpu().double().numpy(), lq=w["teacher_logp"][s:e].cpu().double().numpy(),
                     seq=seq[i:i + 1], lag=w["lag_host"][i:i + 1])
            jobs.append((path, tuple(hp)))
        jobs.sort(key=lambda j: -os.path.getsize(j[0]))     # longest first
        # worker processes are started afresh (never forked from this GPU process); a worker that cannot start
        # raises here instead of being restarted for ever
        with ProcessPoolExecutor(max_workers=cores, mp_context=mp.get_context("spawn")) as pool:
            list(pool.map(_cpu_baseline_worker, [(None, None)] * cores, timeout=120))   # start workers, import numpy
            t0 = time.perf_counter()
            trainable = sum(pool.map(_cpu_baseline_worker, jobs, timeout=600))
            dt = time.perf_counter() - t0
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return dict(value=trainable / dt, unit="tokens/s", cores=cores, kind="oracle",
                sample="%d whole samples (%d rows, V=%d) of the same workload, full pass incl. bf16 gradient, one "
                       "sample per task on %d worker processes: %.1f s wall, numpy float64"
                       % (len(chosen), rows, w["V"], cores, dt))


def bench_full_kl(args, torch, fb, wl, LossPass, hp):
    """One JSON line for the two-tensor variants on the same workload plus a second logits tensor:
    fopd_loss_fwd_bwd_full_kl (second tensor = stale checkpoint) or, with --variant full_teacher,
    fopd_loss_fwd_bwd_full_teacher (second tensor = teacher; the same two kernels)."""
    teacher = args.variant == "full_teacher"
    w = wl.generate(args.workload, "cuda:0", seed=0, stale_logit_sigma=0.03)
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]
    lp = LossPass(T, V, B, w["dtype"], ld=ld, device="cuda:0")
    kl = torch.empty(T, device="cuda:0")

    def step():
        if teacher:
            fb.fopd_loss_fwd_bwd_full_teacher(w["logits"], w["logits_stale"], lp.dt, T, V, ld, ld, w["token_ids"],
                                              w["mask"], w["behav_logp"], w["teacher_logp_stale"], w["seq_lens"],
                                              w["lag"], B, hp, None, None, None, 0, None, None, None, None, 1.0,
                                              lp.loss, lp.freshness, lp.weights, lp.logp, kl, lp.dlogits,
                                              lp.workspace)
        else:
            fb.fopd_loss_fwd_bwd_full_kl(w["logits"], w["logits_stale"], lp.dt, T, V, ld, ld, w["token_ids"],
                                         w["mask"], w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"],
                                         w["lag"], B, hp, None, None, None, 0, None, None, None, None, 1.0, lp.loss,
                                         lp.freshness, lp.weights, lp.logp, kl, lp.dlogits, lp.workspace)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    fb.fopd_profile_reset()
    fb.fopd_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    fb.fopd_profile_enable(False)
    k5_ms, n5 = fb.fopd_profile_read(0)
    k6_ms, n6 = fb.fopd_profile_read(1)
    e = 2 if w["dtype"] == "bf16" else 4
    import numpy as np
    live = int((w["mask_host"] != 0).sum())
    per_row_w = np.repeat(lp.weights.cpu().numpy(), w["seq_lens_host"])
    grad_rows = int(((w["mask_host"] != 0) & (per_row_w > 0)).sum())    # rows of gated samples are zero-filled unread
    k5_bytes = live * 2 * V * e
    k6_bytes = grad_rows * 3 * V * e + (T - grad_rows) * V * e
    k5_s, k6_s = k5_ms / max(n5, 1) * 1e-3, k6_ms / max(n6, 1) * 1e-3
    print(json.dumps({
        "metric": ("tokens/s, OPD loss fwd+bwd with distribution-level loss against teacher logits, V=%d %s"
                   if teacher else "tokens/s, OPD loss fwd+bwd with full-vocabulary rollout KL, V=%d %s")
                  % (V, w["dtype"]),
        "value": w["n_trainable"] * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload + ("+teacher_logits" if teacher else "+stale_logits"), "B": B,
                   "T_rows": T, "V": V, "storage": w["dtype"],
                   "call": "fopd_loss_fwd_bwd_full_teacher" if teacher else "fopd_loss_fwd_bwd_full_kl"},
        "roofline": {"bound": "hbm", "kernel": "fopd_k6_grad_kl", "achieved": k6_bytes / k6_s / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": k6_bytes / k6_s / 1e9 / HBM_PEAK_GBS,
                     "traffic": None, "bytes_per_launch": k6_bytes, "avg_ms": k6_s * 1e3},
        "kernels": {"fopd_k5_kl": {"avg_ms": k5_s * 1e3, "GB/s": k5_bytes / k5_s / 1e9,
                                   "frac": k5_bytes / k5_s / 1e9 / HBM_PEAK_GBS}}}))


def bench_topk_teacher(args, torch, fb, wl, hp):
    """One JSON line for fopd_loss_fwd_bwd_topk_teacher: the bench workload plus a teacher stored as --list-k tokens
    per row.  The two streaming kernels are those of the headline; the list is handled by two small kernels."""
    k = args.list_k
    w = wl.generate(args.workload, "cuda:0", seed=0, teacher_list=(k, 0.5))
    T, V, B, ld = w["T"], w["V"], w["B"], w["ld"]
    dev = "cuda:0"
    f32 = dict(dtype=torch.float32, device=dev)
    dt = fb.FOPD_BF16 if w["dtype"] == "bf16" else fb.FOPD_F32
    loss, fresh, weights = torch.empty(1, **f32), torch.empty(B, **f32), torch.empty(B, **f32)
    logp, token_loss = torch.empty(T, **f32), torch.empty(T, **f32)
    dlogits = torch.empty_like(w["logits"])
    nbytes = fb.fopd_topk_workspace_bytes(T, B, k)
    raw = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    off = (-raw.data_ptr()) % 256
    ws = raw[off:off + nbytes]
    fb.fopd_workspace_init(ws)

    def step():
        fb.fopd_loss_fwd_bwd_topk_teacher(w["logits"], dt, T, V, ld, w["token_ids"], w["mask"], w["behav_logp"],
                                          w["list_ids"], w["list_logp"], k, 1e-4, w["teacher_logp"],
                                          w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp, None, None, None,
                                          0, None, None, 1.0, loss, fresh, weights, logp, token_loss, dlogits, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    fb.fopd_profile_reset()
    fb.fopd_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    fb.fopd_profile_enable(False)
    st, flags = fb.fopd_workspace_status(ws)
    if st != 0 or flags != 0:
        sys.exit("bench.py: device flags %d" % flags)
    k1_ms, n1 = fb.fopd_profile_read(0)
    k4_ms, n4 = fb.fopd_profile_read(1)
    import numpy as np
    e = 2 if w["dtype"] == "bf16" else 4
    live = int((w["mask_host"] != 0).sum())
    per_row_w = np.repeat(weights.cpu().numpy(), w["seq_lens_host"])
    grad_rows = int(((w["mask_host"] != 0) & (per_row_w > 0)).sum())
    k1_bytes = live * V * e
    k4_bytes = grad_rows * 2 * V * e + (T - grad_rows) * V * e
    k1_s, k4_s = k1_ms / max(n1, 1) * 1e-3, k4_ms / max(n4, 1) * 1e-3
    ms = elapsed / args.steps * 1e3
    print(json.dumps({
        "metric": "tokens/s, OPD loss fwd+bwd with distribution-level loss against a teacher stored as %d tokens "
                  "per row, V=%d %s" % (k, V, w["dtype"]),
        "value": w["n_trainable"] * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload + "+teacher_list", "B": B, "T_rows": T, "V": V, "k": k,
                   "storage": w["dtype"], "call": "fopd_loss_fwd_bwd_topk_teacher"},
        "roofline": {"bound": "hbm",
                     "kernel": "fopd_k4_grad_regs" if V // (8 if w["dtype"] == "bf16" else 4) > 2048 else "fopd_k4_grad",
                     "achieved": k4_bytes / k4_s / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": k4_bytes / k4_s / 1e9 / HBM_PEAK_GBS,
                     "traffic": None, "bytes_per_launch": k4_bytes, "avg_ms": k4_s * 1e3},
        "kernels": {"fopd_k1_lse": {"avg_ms": k1_s * 1e3, "GB/s": k1_bytes / k1_s / 1e9,
                                    "frac": k1_bytes / k1_s / 1e9 / HBM_PEAK_GBS},
                    "list kernels, scores, coefficients": {"ms_per_step": ms - (k1_s + k4_s) * 1e3}}}))


MFMA_BF16_PEAK_TFLOPS = 2500.0


def bench_lm_head(args, torch, fb, wl, steps=None):
    """Result record for fopd_lm_head_token_logprobs: log-probs straight from hidden states (d = 4096) and
    the [V, d] output projection, on as many rows as the workload has, with its mask."""
    steps = args.steps if steps is None else steps
    seq_lens, mask = wl.structure_only(args.workload, seed=0)
    T, d, V = int(seq_lens.sum()), 4096, int(wl.CONFIGS[args.workload]["V"])
    w = wl.generate_lm_head(T, d, V, "cuda:0", seed=0)
    w["mask"] = torch.from_numpy(mask).to("cuda:0")
    nbytes = fb.fopd_lm_head_workspace_bytes(T)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda:0")
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + nbytes]
    fb.fopd_workspace_init(ws)
    logp = torch.empty(T, dtype=torch.float32, device="cuda:0")
    lse = torch.empty(T, dtype=torch.float32, device="cuda:0")
    # masked rows are not projected unless --no-compact asks for every row
    fb.fopd_set_option("lm_head_compact", 0 if args.no_compact else 1)
    rows = T if args.no_compact else int((mask != 0).sum())

    def step():
        fb.fopd_lm_head_token_logprobs(w["hidden"], d, w["weight"], d, T, V, d, w["token_ids"], w["mask"],
                                       logp, lse, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    fb.fopd_profile_reset()
    fb.fopd_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    fb.fopd_profile_enable(False)
    st, flags = fb.fopd_workspace_status(ws)
    if st != 0:
        sys.exit("device flags set: %d" % flags)
    k7_ms, n7 = fb.fopd_profile_read(3)
    k7_s = k7_ms / max(n7, 1) * 1e-3
    flops = 2.0 * rows * V * d                          # the rows that are projected
    return {
        "metric": "tokens/s, token log-probs from hidden states (projection fused, logits never stored), "
                  "V=%d d=%d bf16" % (V, d),
        "value": int((mask != 0).sum()) * steps / elapsed, "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": args.warmup, "ms_per_step": elapsed / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload + "+lm_head", "T_rows": T, "rows_with_mask_0": int((mask == 0).sum()),
                   "masked_rows_projected": bool(args.no_compact), "V": V, "d": d,
                   "call": "fopd_lm_head_token_logprobs"},
        "roofline": {"bound": "mfma", "kernel": "fopd_k7_lm_head_lse", "achieved": flops / k7_s / 1e12,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": flops / k7_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None, "flops_per_launch": flops, "avg_ms": k7_s * 1e3}}


def bench_lm_head_loss(args, torch, fb, wl, hp, steps=None, rows_chunk=None, with_listed=False):
    """Result record for fopd_lm_head_loss_fwd_bwd: loss, dL/dhidden and dL/dweight from hidden states (d = 4096),
    the [V, d] projection and scores computed beforehand, on the rows, mask and lags of the workload; the
    logits exist only as one chunk of `rows_chunk` rows at a time."""
    import numpy as np
    steps = args.steps if steps is None else steps
    rows_chunk = args.rows_chunk if rows_chunk is None else rows_chunk
    seq_lens, mask = wl.structure_only(args.workload, seed=0)
    cfg = wl.CONFIGS[args.workload]              # lags over the workload's range (0 .. 4 where it states none)
    lag = np.random.RandomState(0).randint(cfg.get("lag_lo", 0), cfg.get("lag_hi", 4) + 1,
                                           size=len(seq_lens)).astype(np.int32)
    T, d, V, B = int(seq_lens.sum()), 4096, int(cfg["V"]), len(seq_lens)
    w = wl.attach_loss_inputs(wl.generate_lm_head(T, d, V, "cuda:0", seed=0), seq_lens, lag, seed=0,
                              teacher_list=(args.list_k, 0.5) if with_listed else None)
    w["mask"] = torch.from_numpy(mask).to("cuda:0")

    def aligned(nbytes):
        ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda:0")
        off = (-ws.data_ptr()) % 256
        ws = ws[off:off + nbytes]
        fb.fopd_workspace_init(ws)
        return ws

    f32 = dict(dtype=torch.float32, device="cuda:0")
    logp, lse = torch.empty(T, **f32), torch.empty(T, **f32)
    # first loop of Algorithm 1 without logits: log-probs from the fused projection kernel, then the scores
    ws1 = aligned(fb.fopd_lm_head_workspace_bytes(T))
    fb.fopd_lm_head_token_logprobs(w["hidden"], d, w["weight"], d, T, V, d, w["token_ids"], w["mask"], logp, lse, ws1)
    ws2 = aligned(fb.fopd_workspace_bytes(T, B))
    fresh, n_train, n_roll = torch.empty(B, **f32), torch.empty(B, dtype=torch.int32, device="cuda:0"), \
        torch.empty(B, dtype=torch.int32, device="cuda:0")
    fb.fopd_freshness_score(logp, w["behav_logp"], None, None, w["teacher_logp"], None, w["mask"], w["seq_lens"],
                            w["lag"], T, B, hp, None, n_train, n_roll, None, None, None, None, None, fresh, None, ws2)
    del ws1, ws2
    ws = aligned(fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk))
    loss, weights = torch.empty(1, **f32), torch.empty(B, **f32)
    dh, dw = torch.empty(T, d, **f32), torch.empty(V, d, **f32)
    # masked rows are left out of the three contractions, and rows without a gradient (gated samples) out of the two
    # gradient ones, unless --no-compact asks for every row to be projected
    fb.fopd_set_option("lm_head_compact", 0 if args.no_compact else 1)

    def step():
        fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], d, w["weight"], d, T, V, d, w["token_ids"], w["mask"], w["behav_logp"],
                                     w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, fresh, n_train, n_roll, 1.0,
                                     rows_chunk, loss, weights, logp, lse, dh, d, dw, d, 0, ws)

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    fb.fopd_profile_reset()
    fb.fopd_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    fb.fopd_profile_enable(False)
    st, flags = fb.fopd_workspace_status(ws)
    if st != 0:
        sys.exit("device flags set: %d" % flags)
    # scores supplied and no per-row outputs wanted: the samples of weight 0 are left out of the call altogether
    lean = None
    if not args.no_compact:
        def step_lean():
            fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], d, w["weight"], d, T, V, d, w["token_ids"], w["mask"],
                                         w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, fresh,
                                         n_train, n_roll, 1.0, rows_chunk, loss, weights, None, None, dh, d, dw, d, 0, ws)
        step_lean()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(steps):
            step_lean()
        torch.cuda.synchronize()
        lean = (time.perf_counter() - t3) / steps * 1e3
        st, flags = fb.fopd_workspace_status(ws)
        if st != 0:
            sys.exit("device flags set: %d" % flags)
    # the same call with no scores supplied: they are formed inside, per chunk of whole samples, so that a step
    # from hidden states projects once instead of twice (when every sample fits into a chunk; else the call sweeps
    # the rows twice: four contractions per chunk)
    inside = None
    if True:
        def step_inside():
            fb.fopd_lm_head_loss_fwd_bwd(w["hidden"], d, w["weight"], d, T, V, d, w["token_ids"], w["mask"],
                                         w["behav_logp"], w["teacher_logp"], w["seq_lens"], w["lag"], B, hp, None, None,
                                         None, 1.0, rows_chunk, loss, weights, logp, lse, dh, d, dw, d, 0, ws,
                                         seq_lens_host=seq_lens, freshness=fresh)
        step_inside()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            step_inside()
        torch.cuda.synchronize()
        inside = (time.perf_counter() - t1) / steps * 1e3
        st, flags = fb.fopd_workspace_status(ws)
        if st != 0:
            sys.exit("device flags set: %d" % flags)
    # the same with the teacher stored as k tokens per row (distribution-level loss; scores formed inside)
    listed = None
    if with_listed:
        k = args.list_k
        del ws
        wsl = aligned(fb.fopd_lm_head_loss_topk_workspace_bytes(T, V, d, B, rows_chunk, k))

        def step_listed():
            fb.fopd_lm_head_loss_fwd_bwd_topk_teacher(
                w["hidden"], d, w["weight"], d, T, V, d, w["token_ids"], w["mask"], w["behav_logp"], w["list_ids"],
                w["list_logp"], k, 1e-4, None, None, w["seq_lens"], w["lag"], B, hp, seq_lens, 1.0, rows_chunk, loss,
                fresh, weights, logp, lse, None, dh, d, dw, d, 0, wsl)
        step_listed()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(steps):
            step_listed()
        torch.cuda.synchronize()
        listed = (time.perf_counter() - t2) / steps * 1e3
        st, flags = fb.fopd_workspace_status(wsl)
        if st != 0:
            sys.exit("device flags set: %d" % flags)
    n_chunks = (T + rows_chunk - 1) // rows_chunk
    ldz = (V + 63) // 64 * 64
    rp = sum(((min(rows_chunk, T - a) + 63) // 64) * 64 for a in range(0, T, rows_chunk))
    # flops per call: logits, dhidden, dweight contractions.  Every row projected: what is issued, operand padding
    # included; else the live rows' for the logits and, for the two gradient contractions, those of the rows that
    # have a gradient row (the tiles' ragged ends are issued on top and not counted)
    w_host = weights.cpu().numpy()
    row_w = np.repeat(w_host, seq_lens)
    live = int((mask != 0).sum())
    with_grad = int(((mask != 0) & (row_w > 0)).sum())
    if args.no_compact or (live == T and with_grad == T):
        live = with_grad = T
        flops = {4: 2.0 * T * V * d, 5: 2.0 * T * ldz * d, 6: 2.0 * rp * V * d}
    else:
        flops = {4: 2.0 * live * V * d, 5: 2.0 * with_grad * ldz * d, 6: 2.0 * with_grad * V * d}
    names = {4: "logits = hidden . weight^T", 5: "dhidden = dlogits . weight", 6: "dweight += dlogits^T . hidden"}
    kern, tot_ms = {}, 0.0
    for slot in (4, 5, 6):
        ms, n = fb.fopd_profile_read(slot)
        per_call_s = ms / steps * 1e-3
        tot_ms += ms / steps
        kern[names[slot]] = {"ms_per_call": ms / steps, "launches_per_call": n // steps,
                             "TFLOP/s": flops[slot] / per_call_s / 1e12,
                             "frac": flops[slot] / per_call_s / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    all_flops = sum(flops.values())
    return {
        "metric": "tokens/s, OPD loss fwd+bwd through the output projection (dL/dhidden, dL/dweight; logits only "
                  "chunk-wise), V=%d d=%d bf16" % (V, d),
        "value": int(((mask != 0) & (mask != 2)).sum()) * steps / elapsed, "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": args.warmup, "ms_per_step": elapsed / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload + "+lm_head", "T_rows": T, "rows_with_mask_0": int((mask == 0).sum()),
                   "gated_samples": int((w_host == 0).sum()), "rows_of_gated_samples": int((row_w == 0).sum()),
                   "rows_without_a_share_left_out_of_the_contractions": not args.no_compact, "V": V, "d": d,
                   "rows_chunk": rows_chunk, "chunks": n_chunks, "call": "fopd_lm_head_loss_fwd_bwd",
                   "scratch_GB": fb.fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk) / 1e9},
        "roofline": {"bound": "mfma", "kernel": "fopd_gemm_nt, fopd_gemm_tn (three contractions per chunk)",
                     "achieved": all_flops / (tot_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": all_flops / (tot_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "flops_per_launch": all_flops / (3 * n_chunks), "avg_ms": tot_ms / (3 * n_chunks)},
        "kernels": kern,
        "outside_the_contractions_ms": elapsed / steps * 1e3 - tot_ms,
        "scores_supplied_no_row_outputs": None if lean is None else {
            "call": "fopd_lm_head_loss_fwd_bwd with logp = lse = NULL (samples of weight 0 are not projected at all)",
            "ms_per_call": lean, "tokens/s": int(((mask != 0) & (mask != 2)).sum()) / (lean * 1e-3)},
        "scores_formed_inside": None if inside is None else {
            "call": "fopd_lm_head_loss_fwd_bwd with freshness_in = NULL (chunks of whole samples; scoring, loss and both "
                    "gradients with one projection per step)",
            "ms_per_call": inside, "tokens/s": int(((mask != 0) & (mask != 2)).sum()) / (inside * 1e-3)},
        "listed_teacher": None if listed is None else {
            "call": "fopd_lm_head_loss_fwd_bwd_topk_teacher (teacher stored as %d tokens per row; chunks of whole samples, "
                    "one projection per step)" % args.list_k,
            "ms_per_call": listed, "tokens/s": int(((mask != 0) & (mask != 2)).sum()) / (listed * 1e-3)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="reasoning")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-projection", action="store_true",
                    help="skip the projection-fused log-prob measurement reported beside the headline")
    ap.add_argument("--rows-chunk", type=int, default=16384,
                    help="rows per chunk of the loss pass through the projection (--variant lm_head_loss)")
    ap.add_argument("--no-compact", action="store_true",
                    help="lm_head, lm_head_loss: project every row, masked ones included (option lm_head_compact = 0)")
    ap.add_argument("--list-k", type=int, default=64,
                    help="tokens per row of the stored teacher (--variant topk_teacher)")
    ap.add_argument("--variant", choices=("default", "full_kl", "full_teacher", "topk_teacher", "lm_head",
                                          "lm_head_loss"),
                    default="default",
                    help="full_kl: the pass whose rollout drift is the full-vocabulary KL against a second "
                         "(stale-checkpoint) logits tensor; lm_head: token log-probs from hidden states with "
                         "the output projection fused in.  Each is reported as its own line, not the headline")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (the loss pass shards by sample with no "
                 "exchange on the hot path); run it with --gpus 1")

    import torch
    from paper_2605_17862_amd import binding as fb
    from harness import workloads as wl
    from paper_2605_17862_amd.loss_pass import DEFAULT_HPARAMS, LossPass

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    fb.load_library()
    hp = DEFAULT_HPARAMS
    if args.variant in ("full_kl", "full_teacher"):
        return bench_full_kl(args, torch, fb, wl, LossPass, hp)
    if args.variant == "topk_teacher":
        return bench_topk_teacher(args, torch, fb, wl, hp)
    if args.variant == "lm_head":
        print(json.dumps(bench_lm_head(args, torch, fb, wl)))
        return
    if args.variant == "lm_head_loss":
        print(json.dumps(bench_lm_head_loss(args, torch, fb, wl, hp, with_listed=True)))
        return
    w = wl.generate(args.workload, "cuda:0", seed=0)
    T, V, B = w["T"], w["V"], w["B"]
    lp = LossPass(T, V, B, w["dtype"], ld=w["ld"], device="cuda:0")

    for _ in range(args.warmup):
        lp.loss_fwd_bwd(w, hp)
    torch.cuda.synchronize()
    fb.fopd_profile_reset()
    fb.fopd_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        lp.loss_fwd_bwd(w, hp)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    fb.fopd_profile_enable(False)
    st, flags = lp.status()
    if st != 0:
        sys.exit("device flags set: %d" % flags)

    k1_ms, k1_n = fb.fopd_profile_read(0)
    k4_ms, k4_n = fb.fopd_profile_read(1)

    # Reported beside the headline, not part of it: the call a training minibatch makes when the buffer
    # was scored beforehand (scores passed in; one kernel makes both passes over each row).
    f_in = lp.freshness.clone()

    def scored_call():
        fb.fopd_loss_fwd_bwd(w["logits"], lp.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                             w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp, f_in,
                             None, None, 0, None, None, 1.0, lp.loss, None, lp.weights, lp.logp, lp.dlogits,
                             lp.workspace)

    for _ in range(args.warmup):
        scored_call()
    torch.cuda.synchronize()
    fb.fopd_profile_reset()
    fb.fopd_profile_enable(True)
    t1 = time.perf_counter()
    for _ in range(args.steps):
        scored_call()
    torch.cuda.synchronize()
    scored_elapsed = time.perf_counter() - t1
    fb.fopd_profile_enable(False)
    k14_ms, k14_n = fb.fopd_profile_read(2)

    # Also beside the headline: the whole pass (log-probs, scores, weights, loss, gradient rows) with the logits
    # read once.  The rows come out at unit sample weight (dL/dz_t = w_i u_t; the caller folds the weight into
    # the next operation), so this is not the headline's output and is reported separately.
    def unit_call():
        fb.fopd_loss_fwd_bwd_unit(w["logits"], lp.dt, T, V, w["ld"], w["token_ids"], w["mask"], w["behav_logp"],
                                  w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"], w["lag"], B, hp, 1.0,
                                  lp.loss, lp.freshness, lp.weights, lp.logp, lp.dlogits, lp.workspace)

    for _ in range(args.warmup):
        unit_call()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        unit_call()
    torch.cuda.synchronize()
    unit_elapsed = time.perf_counter() - t2
    st, flags = lp.status()
    if st != 0:
        sys.exit("device flags set: %d" % flags)
    # A yardstick that shares nothing with the kernels: the tensor library's device-to-device copy of the same
    # logits into the same gradient buffer, in this process.  (Where the driver placed the pair of buffers moves
    # every copy-shaped kernel by a few per cent; this copy sees the same placement as the gradient kernel did.)
    copy_ms = None
    if lp.dlogits.shape == w["logits"].shape:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        lp.dlogits.copy_(w["logits"])
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            lp.dlogits.copy_(w["logits"])
        e1.record()
        torch.cuda.synchronize()
        copy_ms = e0.elapsed_time(e1) / 5
    ms_per_step = elapsed / args.steps * 1e3
    n_train = w["n_trainable"]

    # algorithmic HBM bytes of one launch (element size e): a live row of an un-gated sample is read
    # once and written once by the gradient kernel; a masked or gated row is only written
    import numpy as np
    e = 2 if w["dtype"] == "bf16" else 4
    wts = lp.weights.cpu().numpy()
    per_row_w = np.repeat(wts, w["seq_lens_host"])
    live = (w["mask_host"] != 0) & (per_row_w > 0)
    rows_live = int(live.sum())
    side = 4 * 4                                        # coef, lse, logp, token id per row
    k4_bytes = rows_live * 2 * V * e + (T - rows_live) * V * e + T * side
    k1_rows = int((w["mask_host"] != 0).sum())
    k1_bytes = k1_rows * V * e + T * (4 + 1 + 8)
    k4_avg_s = k4_ms / max(k4_n, 1) * 1e-3
    k1_avg_s = k1_ms / max(k1_n, 1) * 1e-3
    achieved = k4_bytes / k4_avg_s / 1e9

    # the gradient kernel's launch shape follows the row length (rows of more than 2048 16-byte vectors are held in
    # registers between their loads and their stores)
    k4_name = "fopd_k4_grad_regs" if V // (8 if w["dtype"] == "bf16" else 4) > 2048 else "fopd_k4_grad"
    out = {
        "metric": "tokens/s and %% HBM peak, fused OPD loss fwd+bwd, V=%s %s" % (format(V, ","), w["dtype"]),
        "value": n_train * args.steps / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "B": B, "T_rows": T, "trainable_tokens": n_train, "V": V,
                   "storage": w["dtype"], "hparams": {"alpha": hp[0], "beta": hp[1], "xi": hp[2], "lambda": hp[3]},
                   "gated_samples": int((wts == 0).sum()), "call": "fopd_loss_fwd_bwd (all steps fused)"},
        "roofline": {"bound": "hbm", "kernel": k4_name, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(args.workload, T, V, k4_name + "_traffic_bytes_per_launch"),
                     "bytes_per_launch": k4_bytes, "avg_ms": k4_avg_s * 1e3},
        "kernels": {"fopd_k1_lse": {"avg_ms": k1_avg_s * 1e3, "GB/s": k1_bytes / k1_avg_s / 1e9,
                                    "frac": k1_bytes / k1_avg_s / 1e9 / HBM_PEAK_GBS},
                    k4_name: {"avg_ms": k4_avg_s * 1e3, "GB/s": achieved},
                    "whole_step_GB/s": (k1_bytes + k4_bytes) / (ms_per_step * 1e-3) / 1e9},
    }
    k14_avg_s = k14_ms / max(k14_n, 1) * 1e-3
    out["scores_supplied"] = {
        "call": "fopd_loss_fwd_bwd with freshness_in (kernel fopd_k14_regs: each row is held in registers between "
                "the two passes, the logits cross the memory system once)",
        "ms_per_call": scored_elapsed / args.steps * 1e3, "tokens/s": n_train * args.steps / scored_elapsed,
        "kernel_avg_ms": k14_avg_s * 1e3, "GB/s": k4_bytes / k14_avg_s / 1e9,
        "frac": k4_bytes / k14_avg_s / 1e9 / HBM_PEAK_GBS}
    unit_bytes = k1_rows * 2 * V * e + (T - k1_rows) * V * e + T * side
    out["single_read_unit_rows"] = {
        "call": "fopd_loss_fwd_bwd_unit (whole pass with each logits row read once: log-probs, scores, weights, loss, "
                "and the gradient rows at unit sample weight, dL/dz_t = w_i u_t)",
        "ms_per_call": unit_elapsed / args.steps * 1e3, "tokens/s": n_train * args.steps / unit_elapsed,
        "GB/s": unit_bytes / (unit_elapsed / args.steps) / 1e9,
        "frac": unit_bytes / (unit_elapsed / args.steps) / 1e9 / HBM_PEAK_GBS}
    if copy_ms is not None:
        copy_bytes = 2 * T * w["ld"] * e
        out["copy_yardstick"] = {
            "call": "torch Tensor.copy_ of the logits into the gradient buffer (same two buffers, same process)",
            "ms": copy_ms, "GB/s": copy_bytes / (copy_ms * 1e-3) / 1e9, "frac": copy_bytes / (copy_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "fopd_k4_grad_over_copy": achieved / (copy_bytes / (copy_ms * 1e-3) / 1e9)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, hp)
    if not args.no_projection:
        # beside the headline: the step in front of the path (its own line under --variant lm_head)
        del lp
        rec = bench_lm_head(args, torch, fb, wl, steps=min(args.steps, 5))
        out["projection_fused"] = {"call": rec["config"]["call"], "d": rec["config"]["d"],
                                   "ms_per_call": rec["ms_per_step"], "tokens/s": rec["value"],
                                   "roofline": rec["roofline"]}
        # and the step behind it: loss and gradient carried through the projection (--variant lm_head_loss)
        del rec, w
        rec = bench_lm_head_loss(args, torch, fb, wl, hp, steps=2)
        out["projection_loss"] = {"call": rec["config"]["call"], "d": rec["config"]["d"],
                                  "rows_chunk": rec["config"]["rows_chunk"], "scratch_GB": rec["config"]["scratch_GB"],
                                  "ms_per_call": rec["ms_per_step"], "tokens/s": rec["value"],
                                  "roofline": rec["roofline"], "kernels": rec["kernels"],
                                  "scores_formed_inside": rec["scores_formed_inside"]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
