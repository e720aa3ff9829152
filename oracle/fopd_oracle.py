"""Float64 CPU oracle for the f-OPD loss pass.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the loss pass computes, written from the
paper's definitions (Sec. 4.1 Eq. "kl-diagnostics", Eq. "freshness"; Sec. 4.2 Eq.
"sample-aggregated-loss", the freshness-weighting expectation, the anchored objective;
Appendix Algorithm 1).  It shares no code with the HIP library and must never be imported by
the product package: only the tests, the smoke check and the benchmark's CPU-baseline leg
may call it.

Everything is numpy float64 (integers are numpy int64/int32).  Rows are handled one at a
time by ordinary Python loops; there is no blocking, fusion or re-ordering beyond what the
definitions state.

Readings of the paper that this oracle fixes (the paper leaves them open):

* The token loss ``l`` (Eq. "sample-aggregated-loss") is the sampled-token reverse-KL term
  ``log pi_theta(y) - log pi_teacher(y)``; it is optimised as a score-function (policy
  gradient) term whose advantage ``A = log pi_teacher(y) - log pi_theta(y)`` is held
  constant.
* ``D_i^roll`` (Eq. "kl-diagnostics", first line) is estimated on the sampled token, which
  was drawn from the rollout policy, by ``k(delta) = rho*delta - rho + 1`` with
  ``delta = log pi^t(y) - log pi^{r(i)}(y)`` and ``rho = exp(delta)``; its expectation under
  the rollout policy is KL(pi^t || pi^{r(i)}) and it is never negative.
* ``D_i^sup`` (Eq. "kl-diagnostics", second line) uses the same ``k`` on the teacher's
  current-context minus stale-context log-probability, or is 0 when no stale-context array
  is given (Remark "When the supervision gap is negligible").
* The two aligned sets U_i^roll and U_i^sup (Sec. 4.1) come in one byte per row: 0 = in neither,
  1 = in both (so a plain 0/1 loss mask means "both"), 2 = in U^roll only, 3 = in U^sup only; any other
  non-zero value counts as 1.  D^roll averages over U^roll; D^sup and the token loss over U^sup; a sample
  with either set empty is invalid (Algorithm 1).
* The expectation over the buffer divides by the number of samples B, whether or not a
  sample is gated or invalid (Algorithm 1, anchored minibatch loss).
* Freshness weights are constants in the gradient (Algorithm 1 scores the buffer before the
  minibatch loop).
* A teacher stored as k tokens per row with their log-probabilities (the paper names distribution-level
  teacher supervision but no storage format) gives the token loss as the reverse KL between the two
  distributions coarsened to the k listed tokens plus one event for every other token; the teacher's
  probability of that last event is what its listed tokens leave of 1, not below a floor the caller passes.
  Listing every token gives the full KL; coarsening can only lower it.

Hyper-parameter values are not given by the paper: parity on them is unpinned by the paper
and rests on both sides receiving the same numbers.
"""

import math

import numpy as np


# ----------------------------------------------------------------------------------------
# integer bookkeeping (Sec. 4.1: token length H_i, aligned sets U_i; Algorithm 1 ratios)
# ----------------------------------------------------------------------------------------

def segment_offsets(seq_lens):
    """cu[0] = 0, cu[i+1] = cu[i] + H_i  (H_i: token length of sample i, Sec. 4.1)."""
    seq_lens = np.asarray(seq_lens)
    cu = np.zeros(seq_lens.shape[0] + 1, dtype=np.int64)
    for i in range(seq_lens.shape[0]):
        if int(seq_lens[i]) < 0:
            raise ValueError("negative sequence length")
        cu[i + 1] = cu[i] + int(seq_lens[i])
    return cu


def in_sup_set(m):
    """Row belongs to U^sup (teacher contexts comparable: the token loss and D^sup use it)."""
    return int(m) != 0 and int(m) != 2


def in_roll_set(m):
    """Row belongs to U^roll (replay under the stale policy comparable: D^roll uses it)."""
    return int(m) != 0 and int(m) != 3


def trainable_counts(mask, cu):
    """n_i = |U_i^sup| = number of rows of segment i that carry the token loss (Sec. 4.1, aligned sets)."""
    mask = np.asarray(mask)
    B = cu.shape[0] - 1
    n = np.zeros(B, dtype=np.int32)
    for i in range(B):
        cnt = 0
        for t in range(int(cu[i]), int(cu[i + 1])):
            if in_sup_set(mask[t]):
                cnt += 1
        n[i] = cnt
    return n


def roll_counts(mask, cu):
    """|U_i^roll| = number of rows of segment i on which the rollout drift is measured."""
    mask = np.asarray(mask)
    B = cu.shape[0] - 1
    n = np.zeros(B, dtype=np.int32)
    for i in range(B):
        n[i] = sum(1 for t in range(int(cu[i]), int(cu[i + 1])) if in_roll_set(mask[t]))
    return n


def gather_index(token_ids, ld):
    """Flat element offset of the sampled token y_t inside a [T, ld] row-major matrix."""
    token_ids = np.asarray(token_ids)
    out = np.zeros(token_ids.shape[0], dtype=np.int64)
    for t in range(token_ids.shape[0]):
        out[t] = int(t) * int(ld) + int(token_ids[t])
    return out


# ----------------------------------------------------------------------------------------
# student log-probability of the sampled token (pi_theta^t(. | x_{i,h}) in Eq.
# "kl-diagnostics" and Eq. "sample-aggregated-loss")
# ----------------------------------------------------------------------------------------

def row_logsumexp(z):
    """log sum_v exp(z_v) of one row, shifted by the row maximum."""
    z = np.asarray(z, dtype=np.float64)
    mx = np.max(z)
    return float(mx + np.log(np.sum(np.exp(z - mx))))


def token_logprobs(logits, token_ids, mask=None):
    """Per row t with mask 1: lse_t and lp_t = z_{t,y_t} - lse_t.  Masked rows give 0, 0.

    logits: [T, V] array whose columns are exactly the vocabulary (a caller holding a padded
    [T, ld] matrix slices the first V columns off before calling).
    """
    logits = np.asarray(logits)
    T, V = logits.shape
    lse = np.zeros(T, dtype=np.float64)
    lp = np.zeros(T, dtype=np.float64)
    for t in range(T):
        if mask is not None and mask[t] == 0:
            continue
        y = int(token_ids[t])
        if y < 0 or y >= V:
            raise ValueError("token id out of range at row %d" % t)
        z = logits[t].astype(np.float64)
        lse[t] = row_logsumexp(z)
        lp[t] = z[y] - lse[t]
    return lse, lp


def lm_head_logits(hidden, weight):
    """z_{t,v} = sum_k h_{t,k} * W_{v,k}: the output projection that makes the student's logits from the
    last hidden state (pi_theta^t(. | x) of Eq. "kl-diagnostics" is softmax of this row).  hidden [T, d],
    weight [V, d] (one row per vocabulary entry); both are widened to float64 exactly and the logits are
    not rounded to any storage type."""
    hidden = np.asarray(hidden, dtype=np.float64)
    weight = np.asarray(weight, dtype=np.float64)
    if hidden.ndim != 2 or weight.ndim != 2 or hidden.shape[1] != weight.shape[1]:
        raise ValueError("hidden [T, d] and weight [V, d] must share d")
    return np.matmul(hidden, weight.T)


def lm_head_token_logprobs(hidden, weight, token_ids, mask=None):
    """lse_t and lp_t as in token_logprobs, on logits formed from the hidden states and never stored."""
    return token_logprobs(lm_head_logits(hidden, weight), token_ids, mask)


def lm_head_loss_fwd_bwd(hidden, weight, token_ids, mask, behav_logp, teacher_logp, seq_lens, lag, freshness,
                         xi, lam, grad_scale=1.0):
    """Second loop of Algorithm 1 (weights from scores computed beforehand, anchored loss, gradient) when the
    student's logits are the projection z = hidden . weight^T and are never kept: the gradient is carried
    through the projection to the hidden states and to the projection matrix,
        dL/dhidden[t, :] = sum_v dL/dz[t, v] * weight[v, :],    dL/dweight[v, :] = sum_t dL/dz[t, v] * hidden[t, :].
    The logits stay unrounded (float64 here); the gradient rows dL/dz are rounded to bfloat16, the type the
    path stores them in between its kernels, before the two contractions ("dhidden", "dweight"); the same two
    contractions of the unrounded rows are returned as "dhidden_exact", "dweight_exact".
    freshness: [B] scores from the first loop; the aligned-set counts come from `mask`."""
    hidden = np.asarray(hidden, dtype=np.float64)
    weight = np.asarray(weight, dtype=np.float64)
    z = lm_head_logits(hidden, weight)
    T, V = z.shape
    if mask is None:
        mask = np.ones(T, dtype=np.uint8)
    cu = segment_offsets(seq_lens)
    if int(cu[-1]) != T:
        raise ValueError("sequence lengths do not add up to T")
    for tau in lag:
        if int(tau) < 0:
            raise ValueError("negative lag")
    lse, lp = token_logprobs(z, token_ids, mask)
    delta, rho, adv, k_roll, k_sup = token_terms(lp, behav_logp, teacher_logp, None)
    D_roll, _, ell, _, n = sample_statistics(lp, teacher_logp, k_roll, k_sup, mask, cu)
    _, n_roll, n_valid = roll_coverage(mask, cu)
    w = freshness_weights(np.asarray(freshness, dtype=np.float64), xi, n_valid)
    loss = anchored_loss(w, ell, D_roll, lam)
    coef = grad_coefficients(delta, rho, adv, mask, cu, n, w, lam, grad_scale, n_roll=n_roll)
    g = np.zeros((T, V))
    for t in range(T):
        g[t] = dlogits_row(z[t], int(token_ids[t]), lse[t], coef[t])
    gb = round_to_bf16(g)
    return dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, logits=z, lse=lse, logp=lp, delta=delta, rho=rho, adv=adv,
                D_roll=D_roll, ell=ell, freshness=np.asarray(freshness, dtype=np.float64), weights=w, loss=loss,
                coef=coef, dlogits_exact=g, dlogits=gb,
                dhidden=np.matmul(gb, weight), dweight=np.matmul(gb.T, hidden),
                dhidden_exact=np.matmul(g, weight), dweight_exact=np.matmul(g.T, hidden))


def token_entropy(logits, mask=None):
    """H_t = -sum_v p_v log p_v of softmax(z_t) (the token-level response entropy that App. B logs as a
    monitoring proxy).  Masked rows give 0; entries with p_v = 0 (logit -inf) contribute 0."""
    logits = np.asarray(logits)
    T = logits.shape[0]
    H = np.zeros(T, dtype=np.float64)
    for t in range(T):
        if mask is not None and mask[t] == 0:
            continue
        z = logits[t].astype(np.float64)
        logp = z - row_logsumexp(z)
        p = np.exp(logp)
        H[t] = -float(np.sum(np.where(p > 0.0, p * np.where(p > 0.0, logp, 0.0), 0.0)))
    return H


# ----------------------------------------------------------------------------------------
# per-token drift and advantage terms
# ----------------------------------------------------------------------------------------

def kl_estimator(d):
    """k(d) = e^d * d - e^d + 1, the sampled-token estimator of KL(current || stale) when the
    token was drawn from the stale distribution and d = log current - log stale."""
    d = np.asarray(d, dtype=np.float64)
    r = np.exp(d)
    return r * d - r + 1.0


def token_terms(logp, behav_logp, teacher_logp, teacher_logp_stale=None):
    """delta_t, rho_t, A_t, k^roll_t, k^sup_t for every row (mask is applied later)."""
    lp = np.asarray(logp, dtype=np.float64)
    lb = np.asarray(behav_logp, dtype=np.float64)
    lq = np.asarray(teacher_logp, dtype=np.float64)
    delta = lp - lb                      # log-ratio current student / rollout policy
    rho = np.exp(delta)                  # importance ratio, not clipped
    adv = lq - lp                        # OPD advantage against the teacher
    k_roll = rho * delta - rho + 1.0
    if teacher_logp_stale is None:
        k_sup = np.zeros_like(lp)
    else:
        eps = lq - np.asarray(teacher_logp_stale, dtype=np.float64)
        k_sup = kl_estimator(eps)
    return delta, rho, adv, k_roll, k_sup


# ----------------------------------------------------------------------------------------
# per-sample statistics (Eq. "kl-diagnostics", Eq. "sample-aggregated-loss", Algorithm 1
# alignment ratios)
# ----------------------------------------------------------------------------------------

def sample_statistics(logp, teacher_logp, k_roll, k_sup, mask, cu, token_loss=None):
    """D_i^roll (token mean over U_i^roll), D_i^sup and l_i (token means over U_i^sup),
    cover_i = |U_i^sup| / H_i and n_i = |U_i^sup|.  token_loss: per-row loss values if not the
    sampled-token form lp - lq.

    Samples with either aligned set empty get zeros everywhere (Algorithm 1, invalid-sample branch)."""
    lp = np.asarray(logp, dtype=np.float64)
    lq = np.asarray(teacher_logp, dtype=np.float64)
    B = cu.shape[0] - 1
    D_roll = np.zeros(B)
    D_sup = np.zeros(B)
    ell = np.zeros(B)
    cover = np.zeros(B)
    n = trainable_counts(mask, cu)
    n_roll = roll_counts(mask, cu)
    for i in range(B):
        a, b = int(cu[i]), int(cu[i + 1])
        H = b - a
        if n[i] == 0 or n_roll[i] == 0:
            continue
        rows = [t for t in range(a, b) if in_sup_set(mask[t])]
        rows_roll = [t for t in range(a, b) if in_roll_set(mask[t])]
        D_roll[i] = math.fsum(float(k_roll[t]) for t in rows_roll) / int(n_roll[i])
        D_sup[i] = math.fsum(float(k_sup[t]) for t in rows) / int(n[i])
        if token_loss is None:
            ell[i] = math.fsum(float(lp[t] - lq[t]) for t in rows) / int(n[i])
        else:
            ell[i] = math.fsum(float(token_loss[t]) for t in rows) / int(n[i])
        cover[i] = int(n[i]) / H
    return D_roll, D_sup, ell, cover, n


def roll_coverage(mask, cu):
    """m_i^roll = |U_i^roll| / H_i (0 for an invalid sample), and the validity count min(|U^sup|, |U^roll|),
    which is 0 exactly for the samples Algorithm 1 marks invalid."""
    n = trainable_counts(mask, cu)
    n_roll = roll_counts(mask, cu)
    B = cu.shape[0] - 1
    cover_roll = np.zeros(B)
    for i in range(B):
        if n[i] == 0 or n_roll[i] == 0:
            continue
        cover_roll[i] = int(n_roll[i]) / (int(cu[i + 1]) - int(cu[i]))
    return cover_roll, n_roll, np.minimum(n, n_roll)


# ----------------------------------------------------------------------------------------
# freshness score, aggregates, weights, loss (Eq. "freshness"; Sec. 4.2; Algorithm 1)
# ----------------------------------------------------------------------------------------

def freshness_score(D_roll, D_sup, lag, n_train, alpha, beta):
    """f_i = exp(-(alpha*sqrt(D_i^roll) + beta*sqrt(D_i^sup))) / (tau_i + 1); 0 for an invalid sample
    (n_train[i] = 0: pass min(|U^sup|, |U^roll|) when the two sets differ)."""
    if alpha < 0 or beta < 0:
        raise ValueError("alpha, beta must be non-negative (Eq. freshness)")
    B = len(D_roll)
    f = np.zeros(B)
    for i in range(B):
        if int(lag[i]) < 0:
            raise ValueError("negative lag")
        if int(n_train[i]) == 0:
            f[i] = 0.0
            continue
        surrogate = alpha * math.sqrt(D_roll[i]) + beta * math.sqrt(D_sup[i])
        f[i] = math.exp(-surrogate) / (int(lag[i]) + 1)
    return f


def buffer_aggregates(f, cover, cover_roll=None):
    """(mean freshness, mean roll coverage, mean sup coverage) over all B samples (Sec. 4.2).
    cover is m^sup; cover_roll = None means the two aligned sets coincide."""
    B = len(f)
    fbar = math.fsum(float(x) for x in f) / B
    mbar = math.fsum(float(x) for x in cover) / B
    mroll = mbar if cover_roll is None else math.fsum(float(x) for x in cover_roll) / B
    return np.array([fbar, mroll, mbar])


def freshness_weights(f, xi, n_train):
    """w_i = ReLU(f_i - xi); invalid samples (n_train[i] = 0, see freshness_score) are excluded
    whatever xi is."""
    w = np.zeros(len(f))
    for i in range(len(f)):
        if int(n_train[i]) == 0:
            continue
        w[i] = max(float(f[i]) - xi, 0.0)
    return w


def anchored_loss(w, ell, D_roll, lam):
    """L = B^-1 * sum_i w_i * (l_i + lambda * D_i^roll)   (Algorithm 1, anchored loss)."""
    B = len(w)
    return math.fsum(float(w[i]) * (float(ell[i]) + lam * float(D_roll[i])) for i in range(B)) / B


# ----------------------------------------------------------------------------------------
# full-vocabulary rollout drift: Eq. "kl-diagnostics", first line, as printed (needs the stale
# checkpoint's logits on the same prefixes)
# ----------------------------------------------------------------------------------------

def rollout_kl_full(logits, logits_stale, mask=None):
    """KL(pi^t(.|x_t) || pi^r(.|x_t)) per row from the two logits tensors; also lse of both.
    Masked rows give 0.  Entries whose current probability is 0 contribute 0."""
    logits = np.asarray(logits)
    logits_stale = np.asarray(logits_stale)
    T = logits.shape[0]
    kl = np.zeros(T)
    lse = np.zeros(T)
    lse_stale = np.zeros(T)
    for t in range(T):
        if mask is not None and mask[t] == 0:
            continue
        z = logits[t].astype(np.float64)
        zs = logits_stale[t].astype(np.float64)
        lse[t] = row_logsumexp(z)
        lse_stale[t] = row_logsumexp(zs)
        logp = z - lse[t]
        logq = zs - lse_stale[t]
        p = np.exp(logp)
        kl[t] = float(np.sum(np.where(p > 0.0, p * (np.where(p > 0.0, logp, 0.0) - logq), 0.0)))
    return kl, lse, lse_stale


def dlogits_row_full_kl(z, zs, y, lse_t, lse_stale_t, kl_t, c1_t, c2_t):
    """One gradient row when the anchor is the full-vocabulary KL:
    c1 (p - onehot) + c2 p (log p - log p' - KL_t);  d KL(p||p')/dz_u = p_u (log p_u - log p'_u - KL)."""
    z = np.asarray(z, dtype=np.float64)
    zs = np.asarray(zs, dtype=np.float64)
    if c1_t == 0.0 and c2_t == 0.0:
        return np.zeros_like(z)
    logp = z - lse_t
    p = np.exp(logp)
    g = p * (c1_t + c2_t * ((logp - (zs - lse_stale_t)) - kl_t))
    g[y] -= c1_t
    return g


def fopd_loss_fwd_bwd_full_kl(logits, logits_stale, token_ids, mask, teacher_logp, teacher_logp_stale,
                              seq_lens, lag, alpha, beta, xi, lam, grad_scale=1.0, out_dtype="f32",
                              want_dlogits=True):
    """The whole pass with D_i^roll taken as the token mean of the full-vocabulary KL (Eq.
    "kl-diagnostics" as printed) instead of the sampled-token estimator, in Algorithm 1's order.  The
    anchor term lambda D_i^roll is then differentiated through the full KL."""
    logits = np.asarray(logits)
    T, V = logits.shape
    if mask is None:
        mask = np.ones(T, dtype=np.uint8)
    cu = segment_offsets(seq_lens)
    if int(cu[-1]) != T:
        raise ValueError("sequence lengths do not add up to T")
    lse, lp = token_logprobs(logits, token_ids, mask)
    kl, lse2, lse_stale = rollout_kl_full(logits, logits_stale, mask)
    lq = np.asarray(teacher_logp, dtype=np.float64)
    adv = lq - lp
    if teacher_logp_stale is None:
        k_sup = np.zeros(T)
    else:
        k_sup = kl_estimator(lq - np.asarray(teacher_logp_stale, dtype=np.float64))
    D_roll, D_sup, ell, cover, n = sample_statistics(lp, lq, kl, k_sup, mask, cu)
    cover_roll, n_roll, n_valid = roll_coverage(mask, cu)
    f = freshness_score(D_roll, D_sup, lag, n_valid, alpha, beta)
    agg = buffer_aggregates(f, cover, cover_roll)
    w = freshness_weights(f, xi, n_valid)
    loss = anchored_loss(w, ell, D_roll, lam)
    B = len(n)
    c1 = np.zeros(T)
    c2 = np.zeros(T)
    for i in range(B):
        if int(n_valid[i]) == 0 or w[i] == 0.0:
            continue
        for t in range(int(cu[i]), int(cu[i + 1])):
            if in_sup_set(mask[t]):
                c1[t] = grad_scale * w[i] / (B * int(n[i])) * adv[t]
            if in_roll_set(mask[t]):
                c2[t] = grad_scale * w[i] / (B * int(n_roll[i])) * lam
    res = dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, lse=lse, lse_stale=lse_stale, logp=lp, adv=adv, roll_kl=kl,
               D_roll=D_roll, D_sup=D_sup, ell=ell, cover=cover, cover_roll=cover_roll, freshness=f, agg=agg,
               weights=w, loss=loss, c1=c1, c2=c2)
    if want_dlogits:
        g = np.zeros((T, V))
        for t in range(T):
            g[t] = dlogits_row_full_kl(logits[t], np.asarray(logits_stale)[t], int(token_ids[t]), lse[t],
                                       lse_stale[t], kl[t], c1[t], c2[t])
        res["dlogits_exact"] = g
        res["dlogits"] = round_to_bf16(g) if out_dtype == "bf16" else round_to_f32(g)
    return res


def fopd_loss_fwd_bwd_full_teacher(logits, teacher_logits, token_ids, mask, behav_logp, teacher_logp_stale,
                                   seq_lens, lag, alpha, beta, xi, lam, grad_scale=1.0, out_dtype="f32",
                                   want_dlogits=True):
    """The whole pass with a distribution-level token loss: l_t = KL(pi_theta(.|x_t) || pi_teacher(.|c_t))
    from the teacher's full logits (Eq. "sample-aggregated-loss" with l taken as the reverse KL between the
    two distributions instead of its sampled-token form).  The rollout drift keeps the sampled-token
    estimator.  Gradient: d l_t/dz_u = p_u (log p_u - log q_u - l_t); the anchor contributes
    -lambda rho delta (p - onehot) as in the default path."""
    logits = np.asarray(logits)
    teacher_logits = np.asarray(teacher_logits)
    T, V = logits.shape
    if mask is None:
        mask = np.ones(T, dtype=np.uint8)
    cu = segment_offsets(seq_lens)
    if int(cu[-1]) != T:
        raise ValueError("sequence lengths do not add up to T")
    lse, lp = token_logprobs(logits, token_ids, mask)
    lse_q, lq = token_logprobs(teacher_logits, token_ids, mask)      # teacher log-prob of the sampled token
    tok_kl, _, _ = rollout_kl_full(logits, teacher_logits, mask)     # KL(student || teacher) per row
    delta, rho, _, k_roll, k_sup = token_terms(lp, behav_logp, lq, teacher_logp_stale)
    B = cu.shape[0] - 1
    D_roll, D_sup, ell, cover, n = sample_statistics(lp, lq, k_roll, k_sup, mask, cu, token_loss=tok_kl)
    cover_roll, n_roll, n_valid = roll_coverage(mask, cu)
    f = freshness_score(D_roll, D_sup, lag, n_valid, alpha, beta)
    agg = buffer_aggregates(f, cover, cover_roll)
    w = freshness_weights(f, xi, n_valid)
    loss = anchored_loss(w, ell, D_roll, lam)
    c1, c2 = np.zeros(T), np.zeros(T)
    for i in range(B):
        if int(n_valid[i]) == 0 or w[i] == 0.0:
            continue
        for t in range(int(cu[i]), int(cu[i + 1])):
            if in_roll_set(mask[t]):
                c1[t] = -grad_scale * w[i] / (B * int(n_roll[i])) * lam * rho[t] * delta[t]
            if in_sup_set(mask[t]):
                c2[t] = grad_scale * w[i] / (B * int(n[i]))
    res = dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, lse=lse, lse_stale=lse_q, logp=lp, teacher_logp=lq,
               roll_kl=tok_kl, token_kl=tok_kl, delta=delta, rho=rho, adv=-lam * rho * delta, D_roll=D_roll,
               D_sup=D_sup, ell=ell, cover=cover, cover_roll=cover_roll, freshness=f, agg=agg, weights=w, loss=loss,
               c1=c1, c2=c2)
    if want_dlogits:
        g = np.zeros((T, V))
        for t in range(T):
            g[t] = dlogits_row_full_kl(logits[t], teacher_logits[t], int(token_ids[t]), lse[t], lse_q[t], tok_kl[t],
                                       c1[t], c2[t])
        res["dlogits_exact"] = g
        res["dlogits"] = round_to_bf16(g) if out_dtype == "bf16" else round_to_f32(g)
    return res


# ----------------------------------------------------------------------------------------
# teacher given on k tokens per row (Eq. "sample-aggregated-loss" with a distribution-level l whose teacher
# side is stored as the k most likely tokens and their log-probabilities)
# ----------------------------------------------------------------------------------------

def topk_buckets(V, ids):
    """The slots of a row that name a token (0 <= id < V); any other id marks an unused slot.  The named
    tokens must be distinct."""
    used = [j for j in range(len(ids)) if 0 <= int(ids[j]) < V]
    named = [int(ids[j]) for j in used]
    if len(set(named)) != len(named):
        raise ValueError("the tokens of a row's teacher list must be distinct")
    return used, named


def topk_token_loss_row(z, ids, logq, rest_floor):
    """Reverse KL between the student's distribution softmax(z) and the teacher's, both coarsened to the
    events {token ids[0]}, ..., {token ids[k-1]}, {any other token}: the teacher's probabilities of the k
    tokens are exp(logq) and the last event has what is left of 1, but at least rest_floor.

      l = sum_j P_j (log P_j - logq_j) + P_rest (log P_rest - log Q_rest)

    Returns (l, G) with G[u] = log P_b - log Q_b for the event b that holds token u:
    d l / d z_u = p_u (G[u] - l).  An event of student probability 0 adds 0."""
    z = np.asarray(z, dtype=np.float64)
    V = z.shape[0]
    used, named = topk_buckets(V, ids)
    logp = z - row_logsumexp(z)
    p = np.exp(logp)
    G = np.zeros(V)
    ell = 0.0
    in_list = np.zeros(V, dtype=bool)
    q_listed = 0.0
    for j, u in zip(used, named):
        in_list[u] = True
        q_listed += math.exp(float(logq[j]))
        G[u] = logp[u] - float(logq[j])
        if p[u] > 0.0:
            ell += p[u] * G[u]
    q_rest = max(1.0 - q_listed, float(rest_floor))
    p_rest = float(np.sum(p[~in_list]))
    if p_rest > 0.0:
        g_rest = math.log(p_rest) - math.log(q_rest)
        ell += p_rest * g_rest
        G[~in_list] = g_rest
    return ell, G


def dlogits_row_topk(z, y, ids, logq, rest_floor, c1_t, c2_t):
    """One gradient row of the pass with the teacher given on k tokens:
    c1 (p - onehot) + c2 p (G - l), G and l as in topk_token_loss_row."""
    z = np.asarray(z, dtype=np.float64)
    if c1_t == 0.0 and c2_t == 0.0:
        return np.zeros_like(z)
    ell, G = topk_token_loss_row(z, ids, logq, rest_floor)
    p = np.exp(z - row_logsumexp(z))
    g = p * (c1_t + c2_t * (np.where(p > 0.0, G, 0.0) - ell))
    g[y] -= c1_t
    return g


def fopd_loss_fwd_bwd_topk_teacher(logits, token_ids, mask, behav_logp, topk_ids, topk_logp, rest_floor,
                                   teacher_logp, teacher_logp_stale, seq_lens, lag, alpha, beta, xi, lam,
                                   grad_scale=1.0, out_dtype="f32", want_dlogits=True):
    """The whole pass with a distribution-level token loss against a teacher that is stored as k tokens per row
    (topk_ids [T, k], topk_logp [T, k]): l_t = topk_token_loss_row.  The rollout drift keeps the sampled-token
    estimator; the supervision drift uses the sampled token's teacher log-probabilities when both arrays are
    given (teacher_logp, teacher_logp_stale) and is 0 otherwise.  Steps in Algorithm 1's order."""
    logits = np.asarray(logits)
    T, V = logits.shape
    if mask is None:
        mask = np.ones(T, dtype=np.uint8)
    cu = segment_offsets(seq_lens)
    if int(cu[-1]) != T:
        raise ValueError("sequence lengths do not add up to T")
    lse, lp = token_logprobs(logits, token_ids, mask)
    tok = np.zeros(T)
    for t in range(T):
        if in_sup_set(mask[t]):
            tok[t], _ = topk_token_loss_row(logits[t], topk_ids[t], topk_logp[t], rest_floor)
    lb = np.asarray(behav_logp, dtype=np.float64)
    delta = lp - lb
    rho = np.exp(delta)
    k_roll = kl_estimator(delta)
    if teacher_logp is None or teacher_logp_stale is None:
        k_sup = np.zeros(T)
    else:
        k_sup = kl_estimator(np.asarray(teacher_logp, dtype=np.float64) -
                             np.asarray(teacher_logp_stale, dtype=np.float64))
    B = cu.shape[0] - 1
    D_roll, D_sup, ell, cover, n = sample_statistics(lp, np.zeros(T), k_roll, k_sup, mask, cu, token_loss=tok)
    cover_roll, n_roll, n_valid = roll_coverage(mask, cu)
    f = freshness_score(D_roll, D_sup, lag, n_valid, alpha, beta)
    agg = buffer_aggregates(f, cover, cover_roll)
    w = freshness_weights(f, xi, n_valid)
    loss = anchored_loss(w, ell, D_roll, lam)
    c1, c2 = np.zeros(T), np.zeros(T)
    for i in range(B):
        if int(n_valid[i]) == 0 or w[i] == 0.0:
            continue
        for t in range(int(cu[i]), int(cu[i + 1])):
            if in_roll_set(mask[t]):
                c1[t] = -grad_scale * w[i] / (B * int(n_roll[i])) * lam * rho[t] * delta[t]
            if in_sup_set(mask[t]):
                c2[t] = grad_scale * w[i] / (B * int(n[i]))
    res = dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, lse=lse, logp=lp, token_loss=tok, delta=delta, rho=rho,
               adv=-lam * rho * delta, D_roll=D_roll, D_sup=D_sup, ell=ell, cover=cover, cover_roll=cover_roll,
               freshness=f, agg=agg, weights=w, loss=loss, c1=c1, c2=c2)
    if want_dlogits:
        g = np.zeros((T, V))
        for t in range(T):
            g[t] = dlogits_row_topk(logits[t], int(token_ids[t]), topk_ids[t], topk_logp[t], rest_floor, c1[t], c2[t])
        res["dlogits_exact"] = g
        res["dlogits"] = round_to_bf16(g) if out_dtype == "bf16" else round_to_f32(g)
    return res


def lm_head_loss_fwd_bwd_topk_teacher(hidden, weight, token_ids, mask, behav_logp, topk_ids, topk_logp, rest_floor,
                                      teacher_logp, teacher_logp_stale, seq_lens, lag, alpha, beta, xi, lam,
                                      grad_scale=1.0):
    """fopd_loss_fwd_bwd_topk_teacher on logits that are the projection z = hidden . weight^T and are never kept
    (every step of Algorithm 1, the scores included), with the gradient carried through the projection as in
    lm_head_loss_fwd_bwd: the rows dL/dz are rounded to bfloat16 before the two contractions ("dhidden",
    "dweight"); "dhidden_exact", "dweight_exact" contract the unrounded rows."""
    hidden = np.asarray(hidden, dtype=np.float64)
    weight = np.asarray(weight, dtype=np.float64)
    z = lm_head_logits(hidden, weight)
    res = fopd_loss_fwd_bwd_topk_teacher(z, token_ids, mask, behav_logp, topk_ids, topk_logp, rest_floor,
                                         teacher_logp, teacher_logp_stale, seq_lens, lag, alpha, beta, xi, lam,
                                         grad_scale=grad_scale, out_dtype="bf16", want_dlogits=True)
    g, gb = res["dlogits_exact"], res["dlogits"]
    res.update(logits=z, dhidden=np.matmul(gb, weight), dweight=np.matmul(gb.T, hidden),
               dhidden_exact=np.matmul(g, weight), dweight_exact=np.matmul(g.T, hidden))
    return res


def refresh_decision(agg, kappa_f, kappa_roll, kappa_sup, step, last_refresh_step, min_interval):
    """Adaptive refresh test (Sec. 4.2 refresh condition; App. B rate limit).  Returns (refresh, reasons):
    reasons lists which of "f", "roll", "sup" hold; refresh is True when any holds and at least
    min_interval steps have passed since the last refresh (last_refresh_step None = never)."""
    fbar, mroll, msup = float(agg[0]), float(agg[1]), float(agg[2])
    reasons = []
    if fbar <= kappa_f:
        reasons.append("f")
    if mroll < kappa_roll:
        reasons.append("roll")
    if msup < kappa_sup:
        reasons.append("sup")
    rested = last_refresh_step is None or step - last_refresh_step >= min_interval
    return (len(reasons) > 0 and rested), reasons


# ----------------------------------------------------------------------------------------
# gradient with respect to the logits
# ----------------------------------------------------------------------------------------

def grad_coefficients(delta, rho, adv, mask, cu, n_train, w, lam, grad_scale=1.0, n_samples=None, n_roll=None):
    """c_t = g * w_i / B * ( [t in U^sup] A_t / |U_i^sup|  -  [t in U^roll] lambda * rho_t * delta_t / |U_i^roll| ),
    which for coinciding sets is g * m_t * w_i / (B * n_i) * (A_t - lambda * rho_t * delta_t).

    B is the number of samples of the whole buffer: len(cu) - 1, or `n_samples` when the arrays
    passed in hold only some of the buffer's samples.  n_roll = None: |U^roll| = |U^sup| = n_train.

    d(-A*lp)/dz = A*(p - onehot) with A constant; d(lambda*k(delta))/dlp = lambda*rho*delta,
    and dlp/dz = onehot - p, hence the minus sign on the anchor part."""
    T = len(delta)
    B = cu.shape[0] - 1 if n_samples is None else int(n_samples)
    if n_roll is None:
        n_roll = n_train
    c = np.zeros(T)
    for i in range(cu.shape[0] - 1):
        if int(n_train[i]) == 0 or int(n_roll[i]) == 0 or w[i] == 0.0:
            continue
        for t in range(int(cu[i]), int(cu[i + 1])):
            part = 0.0
            if in_sup_set(mask[t]):
                part += adv[t] / int(n_train[i])
            if in_roll_set(mask[t]):
                part -= lam * rho[t] * delta[t] / int(n_roll[i])
            c[t] = grad_scale * w[i] / B * part
    return c


def dlogits_row(z, y, lse_t, c_t):
    """One row of dLoss/dlogits: c_t * (softmax(z) - onehot(y)) in float64."""
    z = np.asarray(z, dtype=np.float64)
    if c_t == 0.0:
        return np.zeros_like(z)
    g = np.exp(z - lse_t)
    g[y] -= 1.0
    return c_t * g


# ----------------------------------------------------------------------------------------
# rounding to the storage types
# ----------------------------------------------------------------------------------------

def round_to_bf16(x):
    """Round float64 values to the nearest bfloat16 (8-bit significand, fp32 exponent range),
    ties to even, straight from float64; returns float64 holding the bf16 value."""
    x = np.asarray(x, dtype=np.float64)
    out = np.array(x, copy=True)
    fin = np.isfinite(x) & (x != 0.0)
    _, e = np.frexp(x[fin])                 # |x| = m * 2^e with m in [0.5, 1)
    e = np.maximum(e - 1, -126)             # exponent of the leading bit, clamped at subnormals
    quantum = np.ldexp(1.0, e - 7)          # spacing of bf16 numbers in that binade
    r = np.rint(x[fin] / quantum) * quantum
    r = np.where(np.abs(r) >= np.ldexp(1.0, 128), np.copysign(np.inf, r), r)
    out[fin] = r
    return out


def bf16_ulp(x):
    """Spacing of bfloat16 numbers at |x| (float64 in, float64 out)."""
    x = np.abs(np.asarray(x, dtype=np.float64))
    _, e = np.frexp(np.where(x == 0.0, 1.0, x))
    e = np.where(x == 0.0, -126, np.maximum(e - 1, -126))
    return np.ldexp(1.0, e - 7)


def round_to_f32(x):
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------------------
# the whole pass, in Algorithm 1's order
# ----------------------------------------------------------------------------------------

def fopd_loss_fwd_bwd(logits, token_ids, mask, behav_logp, teacher_logp, teacher_logp_stale,
                      seq_lens, lag, alpha, beta, xi, lam, grad_scale=1.0,
                      out_dtype="f32", want_dlogits=True, ld=None, unit_rows=False):
    """Runs every step on whole arrays and returns a dict of all intermediate and final values.

    logits: [T, V] float array (bf16 inputs must be widened exactly by the caller).
    out_dtype: "f32" or "bf16" - the storage type dlogits is rounded to.
    unit_rows: also return the gradient rows at unit sample weight (coef_unit, unit_rows_exact, unit_rows):
    dlogits_exact[t] = weights[i(t)] * unit_rows_exact[t].
    """
    logits = np.asarray(logits)
    T, V = logits.shape
    if mask is None:
        mask = np.ones(T, dtype=np.uint8)
    cu = segment_offsets(seq_lens)
    if int(cu[-1]) != T:
        raise ValueError("sequence lengths do not add up to T")
    gidx = gather_index(token_ids, V if ld is None else ld)
    lse, lp = token_logprobs(logits, token_ids, mask)
    delta, rho, adv, k_roll, k_sup = token_terms(lp, behav_logp, teacher_logp, teacher_logp_stale)
    D_roll, D_sup, ell, cover, n = sample_statistics(lp, teacher_logp, k_roll, k_sup, mask, cu)
    cover_roll, n_roll, n_valid = roll_coverage(mask, cu)
    f = freshness_score(D_roll, D_sup, lag, n_valid, alpha, beta)
    agg = buffer_aggregates(f, cover, cover_roll)
    w = freshness_weights(f, xi, n_valid)
    loss = anchored_loss(w, ell, D_roll, lam)
    coef = grad_coefficients(delta, rho, adv, mask, cu, n, w, lam, grad_scale, n_roll=n_roll)
    res = dict(cu_seqlens=cu, n_train=n, n_roll=n_roll, gather_idx=gidx, lse=lse, logp=lp, delta=delta,
               rho=rho, adv=adv, k_roll=k_roll, k_sup=k_sup, D_roll=D_roll, D_sup=D_sup,
               ell=ell, cover=cover, cover_roll=cover_roll, freshness=f, agg=agg, weights=w, loss=loss, coef=coef)
    if want_dlogits:
        g = np.zeros((T, V), dtype=np.float64)
        for t in range(T):
            g[t] = dlogits_row(logits[t], int(token_ids[t]), lse[t], coef[t])
        res["dlogits_exact"] = g
        res["dlogits"] = round_to_bf16(g) if out_dtype == "bf16" else round_to_f32(g)
    if unit_rows:
        # The weight is a constant of the sample in the gradient (Algorithm 1 applies it to the sample's loss
        # term; Eq. weight is not differentiated), so dL/dz_t = w_i u_t with u_t the row's gradient at w_i = 1:
        # only w_i needs every row of the sample, u_t needs row t alone.  Invalid samples have no loss term.
        ones = np.where(np.asarray(n_valid) > 0, 1.0, 0.0)
        coef_unit = grad_coefficients(delta, rho, adv, mask, cu, n, ones, lam, grad_scale, n_roll=n_roll)
        res["coef_unit"] = coef_unit
        u = np.zeros((T, V), dtype=np.float64)
        for t in range(T):
            u[t] = dlogits_row(logits[t], int(token_ids[t]), lse[t], coef_unit[t])
        res["unit_rows_exact"] = u
        res["unit_rows"] = round_to_bf16(u) if out_dtype == "bf16" else round_to_f32(u)
    return res
