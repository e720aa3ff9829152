/*
 * fopd.h - C ABI of the f-OPD loss pass for AMD MI355X (gfx950).
 *
 * The library evaluates, for one batch of buffered rollouts, the freshness-weighted,
 * rollout-anchored on-policy-distillation objective of the f-OPD paper and its gradient
 * with respect to the student logits:
 *
 *   per token   lp_t   = log softmax(z_t)[y_t]                       (student term of Eq. "kl-diagnostics"
 *                                                                     and Eq. "sample-aggregated-loss")
 *               delta_t = lp_t - lb_t,  rho_t = exp(delta_t)          (log-ratio to the rollout policy)
 *               A_t    = lq_t - lp_t                                  (advantage against the teacher)
 *               k(d)   = e^d d - e^d + 1                              (sampled-token KL estimator)
 *   per sample  D_i^roll = mean_{t in U_i^roll} k(delta_t)            (Eq. "kl-diagnostics", line 1)
 *               D_i^sup  = mean_{t in U_i^sup} k(lq_t - lq_t^stale)   (Eq. "kl-diagnostics", line 2; 0 if absent)
 *               l_i      = mean_{t in U_i^sup} (lp_t - lq_t)          (Eq. "sample-aggregated-loss")
 *               f_i      = exp(-alpha sqrt(D_i^roll) - beta sqrt(D_i^sup)) / (tau_i + 1)   (Eq. "freshness")
 *               w_i      = max(f_i - xi, 0)                           (freshness weighting, Sec. 4.2)
 *   buffer      L = B^-1 sum_i w_i (l_i + lambda D_i^roll)            (anchored objective, Algorithm 1)
 *   gradient    dL/dz_{t,v} = c_t (softmax(z_t)_v - [v = y_t]),
 *               c_t = g w_i / B ( [t in U_i^sup] A_t / |U_i^sup| - [t in U_i^roll] lambda rho_t delta_t / |U_i^roll| ),
 *               w_i and A_t held constant.
 *
 * U_i^roll and U_i^sup are the aligned sets of Sec. 4.1, named row by row by the `mask` argument (see
 * FOPD_ALIGNED_*; a plain 0/1 loss mask makes them coincide), H_i = seq_lens[i], tau_i = lag[i], and a
 * sample with either set empty has f_i = w_i = 0 (Algorithm 1, invalid-sample branch).
 *
 * Conventions common to every entry point
 *   - Every pointer argument is a DEVICE pointer (HIP device memory) unless it is named
 *     "*_host".  The caller owns all buffers; the library allocates no device memory.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  No entry point synchronises, except those documented as host-synchronous.
 *   - The library keeps no state between calls except what fopd_set_option and the fopd_profile_* hooks
 *     set (process-wide, behind one mutex) and a per-device note that a kernel attribute has been set.
 *     The entry points may be called from several threads; calls that share a workspace must be ordered
 *     by the caller (same stream, or events).
 *   - Matrices are row-major [T, ld] with ld >= V; columns V..ld-1 are never read or written.
 *     The base address must be 16-byte aligned and ld * sizeof(element) a multiple of 16.
 *   - The return value reports what the host can check before launching (arguments, sizes,
 *     alignment, workspace size) and launch failures.  Conditions only visible on the device
 *     (token id outside [0, V), negative lag or length, lengths not adding up to T, a mask that names
 *     two different aligned sets where only one count array was passed) set sticky bits in the first
 *     int32 of the workspace; fopd_workspace_status() reads them.  A row with an out-of-range token id
 *     gets lp = lse = 0 and a zero gradient row (its sample still counts it); a sample with a negative lag is treated as invalid (f_i = w_i = 0, both
 *     alignment ratios 0); a row of only one set whose call has no n_roll_in gets a zero gradient row
 *     and adds nothing to the loss.
 *   - Non-finite inputs propagate to non-finite outputs; nothing traps.
 *   - Identical inputs give bit-identical outputs (all reductions have a fixed order).
 *   - Rows in neither aligned set (mask 0) produce lp = lse = 0 and an all-zero gradient row and are not read.
 */
#ifndef FOPD_H
#define FOPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FOPD_OK = 0,
  FOPD_EINVAL = 1,       /* NULL required pointer, negative alpha/beta, inconsistent optional arguments */
  FOPD_ESHAPE = 2,       /* T < 0 or T >= 2^31, V or B <= 0 (T = 0 is allowed and does nothing), ld < V, V > 2^31-16 */
  FOPD_EALIGN = 3,       /* base pointer or row pitch not 16-byte aligned */
  FOPD_EDTYPE = 4,       /* dtype is neither FOPD_F32 nor FOPD_BF16 */
  FOPD_EWORKSPACE = 5,   /* workspace NULL, misaligned (256 B) or smaller than fopd_workspace_bytes */
  FOPD_ETOKEN_RANGE = 6, /* device flag: some token id outside [0, V) */
  FOPD_ESEGMENTS = 7,    /* device flag: seq_lens negative or not covering the rows of the call */
  FOPD_ELAG = 8,         /* device flag: some lag < 0 */
  FOPD_EHIP = 9,         /* a HIP runtime call or kernel launch failed */
  FOPD_ESETS = 10,       /* device flag: mask bytes 2 / 3 (the two aligned sets differ) in a chunk call made without n_roll_in */
  FOPD_ELIMIT = 11,      /* T or B beyond the fixed limits of an entry point that owns its scratch memory */
  FOPD_STATUS_ANY_INT = 0x7fffffff   /* not a status: makes every int a value of the type, so that a caller's
                                        out-of-range code reaches fopd_status_string's default branch defined */
} fopd_status;

/* (FOPD_DTYPE_ANY_INT is not an element type: with it a caller's unknown code is a value of the type, which the
 * entry points answer with FOPD_EDTYPE) */
typedef enum { FOPD_F32 = 0, FOPD_BF16 = 1, FOPD_DTYPE_ANY_INT = 0x7fffffff } fopd_dtype;

/* Hyper-parameters of Algorithm 1: score coefficients alpha, beta >= 0 (Eq. "freshness"),
 * gate threshold xi (freshness weighting) and anchor strength lambda (full objective). */
typedef struct {
  float alpha;
  float beta;
  float xi;
  float lambda;
} fopd_hparams;

/* Static, NUL-terminated description of a status code. Never NULL. */
const char* fopd_status_string(fopd_status status);

/* Bytes of device workspace that any entry point needs for a call with at most T rows and B
 * samples (a multiple of 256).  The workspace must be 256-byte aligned. */
size_t fopd_workspace_bytes(int64_t T, int32_t B);

/* Clears the sticky device flags at the head of a workspace (asynchronous, on `stream`).
 * Must be called once before the first use of a workspace; may be called again at any time. */
fopd_status fopd_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* HOST-SYNCHRONOUS.  Waits for `stream`, reads the sticky device flags and returns FOPD_OK or the
 * first of FOPD_ETOKEN_RANGE, FOPD_ESEGMENTS, FOPD_ELAG, FOPD_ESETS that is set.  If flags_host is not
 * NULL it receives the raw bit mask (bit 0 token range, bit 1 segments, bit 2 lag, bit 3 aligned sets). */
fopd_status fopd_workspace_status(const void* workspace, void* stream, int32_t* flags_host);

/* HOST ONLY.  The status that a raw flag word (as above) stands for. */
fopd_status fopd_flags_status(int32_t flags);

/*
 * The `mask` argument of every entry point: one byte per row naming the aligned sets of Sec. 4.1 that
 * the row belongs to.  U^roll (replay under the stale policy is comparable) carries the rollout drift
 * D^roll; U^sup (the teacher's contexts are comparable) carries the token loss and the supervision
 * drift D^sup.  A plain 0/1 loss mask puts every kept row in both sets.  A sample with either set
 * empty is invalid (Algorithm 1): f_i = w_i = 0, both alignment ratios 0, zero gradient rows.
 * Any other non-zero byte counts as FOPD_ALIGNED_BOTH; mask == NULL means all rows in both sets.
 */
enum {
  FOPD_ALIGNED_NONE = 0,   /* in neither set: nothing is computed for the row, its gradient row is zero */
  FOPD_ALIGNED_BOTH = 1,
  FOPD_ALIGNED_ROLL = 2,   /* in U^roll only */
  FOPD_ALIGNED_SUP = 3     /* in U^sup only */
};

/*
 * Student log-probability of the sampled tokens: the streaming pass over the logits.
 * (pi_theta^t(y_{i,h} | x_{i,h}) of Eq. "kl-diagnostics" / Eq. "sample-aggregated-loss".)
 *
 *   logits      [T, ld] of `dt`, read once (masked rows are skipped)
 *   token_ids   [T] int32, sampled token y_t of each row
 *   mask        [T] uint8 0/1, NULL = all ones
 *   logp        [T] f32 out: lp_t = z_{t,y_t} - lse_t   (0 for masked rows)
 *   lse         [T] f32 out: log sum_v exp(z_{t,v})      (0 for masked rows)
 *   gather_idx  [T] int64 out, NULL to skip: t * ld + y_t for every row, masked or not (an element
 *               offset from the `logits` pointer of this call)
 *   entropy     [T] f32 out, NULL to skip: H_t = -sum_v p_v log p_v of softmax(z_t), the token-level
 *               response entropy logged as a monitoring proxy (App. B); 0 for masked rows.  Costs
 *               one more multiply-add per logit in the same pass, no extra memory traffic.
 *
 * lp_t is formed from the sum over v != y_t, so it keeps full relative accuracy as
 * softmax(z_t)[y_t] approaches 1.
 */
fopd_status fopd_token_logprobs(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                const int32_t* token_ids, const uint8_t* mask,
                                float* logp, float* lse, int64_t* gather_idx, float* entropy,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Per-sample drift diagnostics and freshness scores (first loop of Algorithm 1; Eq.
 * "kl-diagnostics", Eq. "freshness", buffer aggregates of Sec. 4.2).  Touches only the
 * per-token and per-sample arrays, never the logits.
 *
 *   logp, behav_logp, teacher_logp  [T] f32: current student, rollout-time student and
 *                                   current-context teacher log-probability of y_t
 *   roll_kl                         [T] f32 or NULL: per-row full-vocabulary KL(pi^t || pi^r) from
 *                                   fopd_rollout_kl; when given it is the token drift that D^roll
 *                                   averages and behav_logp is not read (it may then be NULL)
 *   token_loss                      [T] f32 or NULL: a per-row token loss computed elsewhere (the
 *                                   distribution-level KL against the teacher's logits, the `roll_kl`
 *                                   output of fopd_rollout_kl called with the teacher's tensor); when
 *                                   given, ell averages it instead of lp - lq, and teacher_logp may be NULL
 *                                   if teacher_logp_stale is NULL too (nothing reads it then)
 *   teacher_logp_stale              [T] f32 or NULL: teacher log-probability under the context
 *                                   used at grading time; NULL gives D^sup = 0
 *   mask [T] uint8 or NULL; seq_lens [B] int32 (sum must be T); lag [B] int32 >= 0
 *   outputs: cu_seqlens [B+1] int64 (exclusive scan of seq_lens),
 *            n_train [B] int32 = |U_i^sup|, n_roll [B] int32 = |U_i^roll|,
 *            D_roll (token mean over U^roll), D_sup and ell (token means over U^sup),
 *            cover = |U_i^sup| / H_i, cover_roll = |U_i^roll| / H_i (both 0 for an invalid sample),
 *            freshness: [B] f32 each,
 *            agg [3] f32 = mean_i f_i, mean_i cover_roll_i, mean_i cover_i.
 *   Any of the output pointers except freshness may be NULL.
 */
fopd_status fopd_freshness_score(const float* logp, const float* behav_logp, const float* roll_kl,
                                 const float* token_loss,
                                 const float* teacher_logp, const float* teacher_logp_stale,
                                 const uint8_t* mask, const int32_t* seq_lens, const int32_t* lag,
                                 int64_t T, int32_t B, fopd_hparams hp,
                                 int64_t* cu_seqlens, int32_t* n_train, int32_t* n_roll,
                                 float* D_roll, float* D_sup, float* ell, float* cover, float* cover_roll,
                                 float* freshness, float* agg,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Loss and gradient (second loop of Algorithm 1), fused with the two steps above when their
 * results are not supplied.
 *
 * The call covers rows [row_begin, row_begin + T) of the concatenation of the B samples.
 *
 *   freshness_in == NULL : everything is computed here; requires lse_in == logp_in ==
 *                          n_train_in == NULL, row_begin == 0 and sum(seq_lens) == T.
 *   freshness_in != NULL : [B] scores computed earlier (Algorithm 1 scores the buffer before
 *                          the minibatch loop); they define the weights.  n_train_in is the
 *                          [B] count array of fopd_freshness_score, or NULL when the call
 *                          covers whole samples (row_begin == 0, sum(seq_lens) == T) and the
 *                          counts are to be taken from `mask`.  n_roll_in: the [B] n_roll array of
 *                          fopd_freshness_score, or NULL when the two sets coincide (a 0/1 mask);
 *                          only with n_train_in.  (n_train_in without n_roll_in on a mask that does hold
 *                          bytes 2 or 3 raises the FOPD_ESETS flag and drops those rows.)
 *                          Without lse_in one kernel makes both passes over each row: with the row held in
 *                          registers when it fits (see fopd_set_option "k14_regs"), so that the logits are read
 *                          from memory once, else re-reading it right after the first pass.
 *   lse_in / logp_in     : both or neither.  When given ([T] f32, the outputs of
 *                          fopd_token_logprobs for these rows) the logits are read only by the
 *                          gradient pass.  Requires freshness_in.
 *
 *   grad_scale  upstream scale g of the loss (1 for the plain objective)
 *   loss        [1] f32 out: sum over the rows of the call of
 *               w_i / B ( [t in U^sup] (lp_t - lq_t) / |U_i^sup| + [t in U^roll] lambda k(delta_t) / |U_i^roll| );
 *               equals L when the call covers all rows, and the chunk's additive share of L otherwise
 *   freshness   [B] f32 out or NULL (a copy of freshness_in when that is given)
 *   weights     [B] f32 out or NULL
 *   logp        [T] f32 out or NULL
 *   dlogits     [T, ld] of `dt` out, rounded to nearest-even; MAY alias `logits` (in place)
 */
fopd_status fopd_loss_fwd_bwd(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                              const int32_t* token_ids, const uint8_t* mask,
                              const float* behav_logp, const float* teacher_logp,
                              const float* teacher_logp_stale,
                              const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp,
                              const float* freshness_in, const int32_t* n_train_in, const int32_t* n_roll_in,
                              int64_t row_begin, const float* lse_in, const float* logp_in,
                              float grad_scale,
                              float* loss, float* freshness, float* weights, float* logp,
                              void* dlogits,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same pass with the logits read once: gradient rows at unit sample weight.
 *
 * In dL/dz_t = c_t (softmax(z_t) - onehot(y_t)) only the factor w_i of c_t (Eq. "weight", a constant of the
 * sample in the gradient: Algorithm 1 applies it to the sample's loss term) needs every row of the sample; the
 * rest, u_t = g / B ( [t in U^sup] A_t / |U_i^sup| - [t in U^roll] lambda rho_t delta_t / |U_i^roll| )
 * (softmax(z_t) - onehot(y_t)), needs row t alone.  fopd_loss_fwd_bwd therefore reads the logits twice (log-probs,
 * then scores, then gradient); this call reads each row once, writes u_t and returns the weights:
 *     dL/dz_t = weights[i(t)] * unit_rows[t].
 * The caller applies the row scale where it is cheapest: it commutes with whatever consumes the rows next (the
 * output projection's backward contractions: scale the [T, d] result or operand instead of the [T, V] rows).
 * A gated sample (w_i = 0 < f_i) has non-zero unit rows and weight 0; an invalid sample (an aligned set empty,
 * negative lag) has zero rows.  loss, freshness, weights and logp are those of fopd_loss_fwd_bwd on the same
 * inputs, formed by the same kernels from these log-probs (which come from the 1024-lane row partition when the
 * row is held in registers, see fopd_set_option "k14_regs": last-place differences from fopd_token_logprobs).
 * Whole samples only (sum(seq_lens) == T).  Rows too long for the registers (more than 19456 16-byte vectors)
 * are read twice by this call too, the second time right after the first.
 *   arguments as in fopd_loss_fwd_bwd; unit_rows [T, ld] of `dt` out, MAY alias `logits`
 */
fopd_status fopd_loss_fwd_bwd_unit(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                   const int32_t* token_ids, const uint8_t* mask,
                                   const float* behav_logp, const float* teacher_logp,
                                   const float* teacher_logp_stale,
                                   const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp,
                                   float grad_scale,
                                   float* loss, float* freshness, float* weights, float* logp,
                                   void* unit_rows,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * fopd_loss_fwd_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving / training loops, harnesses that forbid allocation.  Same arguments, modes, kernels
 * and results (bit for bit) as fopd_loss_fwd_bwd, except that the scratch memory is an array inside the
 * library (about 1.3 MB of device memory per GPU, held from module load until the process ends) and
 * therefore
 *   - T <= FOPD_STATIC_MAX_ROWS and B <= FOPD_STATIC_MAX_SAMPLES, else FOPD_ELIMIT and nothing is launched
 *     (long buffers go through it chunk by chunk, exactly like the chunked flow of fopd_loss_fwd_bwd);
 *   - the sticky device flags live in that array too: they are cleared at the start of every call and, if
 *     flags_out (a DEVICE int32, may be NULL) is given, copied there at the end (fopd_flags_status decodes them);
 *   - every call on one GPU uses that GPU's one array: calls that may overlap on a GPU (different streams
 *     without an ordering between them, several host threads) race and must be serialised by the caller.
 * The call allocates nothing, frees nothing, records no memset and creates no event (the fopd_profile_* hooks
 * do not see it).  The first call on a device looks the array's address up (and, when freshness_in is given
 * without lse_in, sets a kernel attribute): make one call outside any stream capture first.
 */
#define FOPD_STATIC_MAX_ROWS 32768
#define FOPD_STATIC_MAX_SAMPLES 4096
fopd_status fopd_loss_fwd_bwd_static(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                     const int32_t* token_ids, const uint8_t* mask,
                                     const float* behav_logp, const float* teacher_logp,
                                     const float* teacher_logp_stale,
                                     const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp,
                                     const float* freshness_in, const int32_t* n_train_in, const int32_t* n_roll_in,
                                     int64_t row_begin, const float* lse_in, const float* logp_in,
                                     float grad_scale,
                                     float* loss, float* freshness, float* weights, float* logp,
                                     void* dlogits, int32_t* flags_out, void* stream);

/*
 * Full-vocabulary rollout drift, Eq. "kl-diagnostics" first line as printed: per row
 *   roll_kl_t = KL( softmax(z_t) || softmax(z'_t) ),   z' = logits of the stale checkpoint pi^{r(i)}
 * replayed on the same prefixes.  One pass over both tensors (masked rows are not read).
 *   logits, logits_stale  [T, ld] / [T, ld_stale] of `dt`
 *   roll_kl, logp, lse    [T] f32 out as in fopd_token_logprobs (0 for masked rows)
 *   dlse                  [T] f32 out: lse_t - lse'_t
 *   logq                  [T] f32 out or NULL: log softmax(z'_t)[y_t], the second tensor's log-probability of
 *                         the sampled token
 * Feed roll_kl to fopd_freshness_score to score the buffer with the paper's own diagnostic.  The two rows
 * may be arbitrarily far apart (each has its own running reference); for close rows the KL, a quantity much
 * smaller than either log-sum-exp, is accumulated directly and keeps ~1e-5 relative accuracy.
 * The same call on the TEACHER's logits gives the distribution-level token loss KL(student || teacher) per
 * row and, in logq, the teacher's log-probability of y_t.
 */
fopd_status fopd_rollout_kl(const void* logits, const void* logits_stale, fopd_dtype dt, int64_t T, int64_t V,
                            int64_t ld, int64_t ld_stale, const int32_t* token_ids, const uint8_t* mask,
                            float* roll_kl, float* logp, float* lse, float* dlse, float* logq,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * The whole pass with D_i^roll = token mean of that full-vocabulary KL, everything computed in the call
 * (segment offsets, log-probs, drift, scores, weights, loss, gradient).  The anchor term lambda D_i^roll is
 * differentiated through the full KL:
 *   dL/dz_{t,u} = c1_t (p_u - [u = y_t]) + c2_t p_u (log p_u - log p'_u - roll_kl_t),
 *   c1_t = g [t in U^sup] w_i / (B |U_i^sup|) A_t,   c2_t = g [t in U^roll] w_i / (B |U_i^roll|) lambda.
 * Arguments as in fopd_loss_fwd_bwd; behav_logp is not needed.  logp, roll_kl, freshness, weights may be
 * NULL.  dlogits may alias logits but not logits_stale.
 *
 *   freshness_in == NULL : whole samples, everything computed here (sum(seq_lens) == T; the other *_in
 *                          arguments NULL, row_begin 0).
 *   freshness_in != NULL : the chunked long-horizon flow, when three [T, V] tensors do not fit.  Per chunk
 *                          fopd_rollout_kl (-> roll_kl, logp, lse, dlse slices), once fopd_freshness_score
 *                          with that roll_kl (-> freshness, n_train, n_roll), then per chunk this call with
 *                          rows [row_begin, row_begin + T): freshness_in [B], n_train_in [B] (required),
 *                          n_roll_in [B] (NULL = the two sets coincide), and the chunk's slices lse_in,
 *                          logp_in, dlse_in, roll_kl_in [T] (all required).  Only coefficients, the chunk's
 *                          additive share of the loss and the gradient rows are made; chunks may cut samples.
 */
fopd_status fopd_loss_fwd_bwd_full_kl(const void* logits, const void* logits_stale, fopd_dtype dt, int64_t T,
                                      int64_t V, int64_t ld, int64_t ld_stale, const int32_t* token_ids,
                                      const uint8_t* mask, const float* teacher_logp,
                                      const float* teacher_logp_stale, const int32_t* seq_lens, const int32_t* lag,
                                      int32_t B, fopd_hparams hp,
                                      const float* freshness_in, const int32_t* n_train_in, const int32_t* n_roll_in,
                                      int64_t row_begin, const float* lse_in, const float* logp_in,
                                      const float* dlse_in, const float* roll_kl_in, float grad_scale,
                                      float* loss, float* freshness, float* weights, float* logp, float* roll_kl,
                                      void* dlogits, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The whole pass with a distribution-level token loss (Eq. "sample-aggregated-loss" with l taken as the
 * reverse KL between the two distributions): l_t = KL( softmax(z_t) || softmax(q_t) ), q = the teacher's
 * full logits under the current context.  The rollout drift keeps the sampled-token estimator on
 * behav_logp; the teacher's log-probability of y_t, needed for D^sup when teacher_logp_stale is given,
 * is taken from teacher_logits.
 *   dL/dz_{t,u} = c1_t (p_u - [u = y_t]) + c2_t p_u (log p_u - log q_u - l_t),
 *   c1_t = -g [t in U^roll] w_i / (B |U_i^roll|) lambda rho_t delta_t,   c2_t = g [t in U^sup] w_i / (B |U_i^sup|).
 * Averaged over y ~ softmax(z) the default path's sampled-token gradient equals this one's KL part.
 *   token_kl  [T] f32 out or NULL: l_t.  Other arguments as in fopd_loss_fwd_bwd_full_kl.
 * dlogits may alias logits but not teacher_logits.
 * Chunked flow (freshness_in != NULL): per chunk fopd_rollout_kl on (logits, teacher_logits) with logq
 * (-> token_kl, logp, lse, dlse, logq slices); once fopd_freshness_score(logp, behav_logp, NULL, token_kl,
 * logq as teacher_logp, ...); then per chunk this call with freshness_in, n_train_in, n_roll_in, row_begin and
 * the slices lse_in, logp_in, dlse_in, token_kl_in, exactly as for fopd_loss_fwd_bwd_full_kl.
 */
fopd_status fopd_loss_fwd_bwd_full_teacher(const void* logits, const void* teacher_logits, fopd_dtype dt, int64_t T,
                                           int64_t V, int64_t ld, int64_t ld_teacher, const int32_t* token_ids,
                                           const uint8_t* mask, const float* behav_logp,
                                           const float* teacher_logp_stale, const int32_t* seq_lens,
                                           const int32_t* lag, int32_t B, fopd_hparams hp,
                                           const float* freshness_in, const int32_t* n_train_in,
                                           const int32_t* n_roll_in, int64_t row_begin, const float* lse_in,
                                           const float* logp_in, const float* dlse_in, const float* token_kl_in,
                                           float grad_scale,
                                           float* loss, float* freshness, float* weights, float* logp, float* token_kl,
                                           void* dlogits, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The whole pass with a distribution-level token loss against a teacher that is stored as k tokens per row with
 * their log-probabilities, instead of a [T, V] tensor of teacher logits (Eq. "sample-aggregated-loss" with l a
 * KL between distributions; the paper names distribution-level teacher supervision and no storage format, so the
 * coarsening below is this library's reading).  Both distributions are reduced to the k + 1 events {listed token
 * 1}, ..., {listed token k}, {any other token}:
 *   P_j = softmax(z_t)[id_j],  P_rest = 1 - sum_j P_j;   Q_j = exp(lq_j),  Q_rest = max(1 - sum_j Q_j, rest_floor)
 *   l_t = sum_j P_j (log P_j - lq_j) + P_rest (log P_rest - log Q_rest)          (an event with P = 0 adds 0)
 * Listing every token gives the full KL( softmax(z_t) || teacher ); merging tokens into the rest can only lower it.
 *   dL/dz_{t,u} = c1_t (p_u - [u = y_t]) + c2_t p_u (G_u - l_t),   G_u = log P_b - log Q_b of the event b holding u,
 *   c1_t = -g [t in U^roll] w_i / (B |U_i^roll|) lambda rho_t delta_t,   c2_t = g [t in U^sup] w_i / (B |U_i^sup|).
 * The rollout drift keeps the sampled-token estimator on behav_logp.  The logits are read twice and the gradient
 * written once, as in fopd_loss_fwd_bwd; the k listed entries per row are gathered and corrected by two small
 * kernels.
 *   list_ids   [T, k] int32  the listed tokens of each row, distinct; an id outside [0, V) marks an unused slot
 *   list_logp  [T, k] f32    their teacher log-probabilities (<= 0; unused slots are ignored)
 *   k          1 .. 4096;  rest_floor in (0, 1]: the least probability the teacher keeps for "any other token"
 *   teacher_logp, teacher_logp_stale  [T] f32 or NULL: the sampled token's teacher log-probabilities under the
 *              current and the stale context, for D^sup only; D^sup = 0 unless both are given
 *              (teacher_logp_stale without teacher_logp is FOPD_EINVAL)
 *   loss [1], freshness [B] or NULL, weights [B] or NULL, logp [T] or NULL, token_loss [T] or NULL (l_t; 0 outside
 *   U^sup): f32 outputs; dlogits [T, ld] in the logits' type, may alias logits
 *   workspace  fopd_topk_workspace_bytes(T, B, k) bytes, 256-byte aligned, initialised once with
 *              fopd_workspace_init; sticky flags as in fopd_loss_fwd_bwd
 * A row whose listed ids repeat a token has an undefined loss and gradient at that token (not checked).
 *
 * Modes, by which of the optional inputs are given (any other combination is FOPD_EINVAL):
 *   none of them        a whole batch: seq_lens add up to T, everything is computed in the call
 *   freshness_in given  a chunk of a longer batch, rows [row_begin, row_begin + T): freshness_in [B], n_train_in
 *                       [B] (required), n_roll_in [B] (NULL = the two sets coincide), and the chunk's slices lse_in,
 *                       logp_in [T] (required).  The flow: per chunk fopd_token_logprobs (-> logp, lse) and
 *                       fopd_topk_token_loss (-> token_loss); once fopd_freshness_score(logp, behav_logp, NULL,
 *                       token_loss, teacher_logp, teacher_logp_stale, ...) over the O(T) arrays; then per chunk this
 *                       call, which forms the listed terms again from lse_in (O(T k)) and makes coefficients, the
 *                       chunk's additive share of the loss and the gradient rows.  Chunks may cut samples; seq_lens
 *                       and lag describe the whole batch; teacher_logp / teacher_logp_stale are not read.
 *
 * fopd_topk_token_loss: l_t alone, for the flow above.  lse [T] f32 from fopd_token_logprobs on the same rows;
 * token_loss [T] f32 out (0 outside U^sup).  Needs no workspace.
 */
size_t fopd_topk_workspace_bytes(int64_t T, int32_t B, int32_t k);
fopd_status fopd_topk_token_loss(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                 const int32_t* token_ids, const uint8_t* mask, const int32_t* list_ids,
                                 const float* list_logp, int32_t k, float rest_floor, const float* lse,
                                 float* token_loss, void* stream);
fopd_status fopd_loss_fwd_bwd_topk_teacher(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                           const int32_t* token_ids, const uint8_t* mask, const float* behav_logp,
                                           const int32_t* list_ids, const float* list_logp, int32_t k,
                                           float rest_floor, const float* teacher_logp,
                                           const float* teacher_logp_stale, const int32_t* seq_lens,
                                           const int32_t* lag, int32_t B, fopd_hparams hp, const float* freshness_in,
                                           const int32_t* n_train_in, const int32_t* n_roll_in, int64_t row_begin,
                                           const float* lse_in, const float* logp_in, float grad_scale, float* loss,
                                           float* freshness, float* weights, float* logp, float* token_loss,
                                           void* dlogits, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Adaptive refresh test (Sec. 4.2, refresh condition; Algorithm 1, step after the aggregates; App. B:
 * the rule may fire at most once every `min_interval` optimizer steps, 200 in the paper).  HOST ONLY: all
 * pointers are host pointers and nothing touches the GPU.  `agg_host` is a host copy of the `agg` output
 * of fopd_freshness_score: mean freshness, mean roll coverage, mean sup coverage.
 *
 * The buffer is to be refreshed when   agg[0] <= kappa_f  or  agg[1] < kappa_roll  or  agg[2] < kappa_sup
 * and no refresh happened in the last `min_interval - 1` steps (last_refresh_step < 0 means never).
 * Returns 1 (refresh: the state records `step` and counts it) or 0; `reason_host`, if not NULL, receives
 * the bits of the conditions that hold (1 freshness, 2 roll coverage, 4 sup coverage) whether or not
 * the rate limit lets the refresh through.  Returns -1 on a NULL argument or min_interval < 1.
 */
typedef struct {
  float kappa_f;
  float kappa_roll;
  float kappa_sup;
  int64_t min_interval;
} fopd_refresh_config;

typedef struct {
  int64_t last_refresh_step; /* initialise to -1 */
  int64_t refreshes;         /* initialise to 0 */
} fopd_refresh_state;

int fopd_refresh_decide(const float* agg_host, const fopd_refresh_config* cfg_host, fopd_refresh_state* state_host,
                        int64_t step, int32_t* reason_host);

/*
 * Launch-shape options (process-wide; a call reads them once, under the library's mutex, when it starts):
 *   "k14_threads"      256, 512 or 1024 lanes per row in the kernel that makes both passes over a row
 *                      (used when freshness_in is given without lse_in); default 256
 *   "k14_rows_per_cu"  1..8 rows in flight per compute unit in that kernel; default 6.
 *   "k14_regs"         1 (default): in that same call, a row of 2049 .. 19456 16-byte vectors (bf16: 16,392 <= V <=
 *                      155,648; fp32: half that) is held in registers between the two passes by a workgroup of
 *                      1024 lanes, so that the logits cross the memory system once; 0: always the kernel above.
 *                      The 1024-lane partition sums a row in another order than fopd_token_logprobs does, so
 *                      log-probs may differ from that call's in the last place.
 *   "k14_regs_grid"    workgroups of that row-in-registers kernel, each walking rows in steps of the grid: 1..4096,
 *                      or 0 (default) for two per compute unit (one is resident at a time; the second half is
 *                      handed out as compute units finish).  The results do not depend on it.
 *   "k4_regs"          1 (default): the gradient kernel of the calls that read the logits twice takes the launch
 *                      shape of the row-in-registers kernel for rows of more than 2048 16-byte vectors (a compute
 *                      unit reads a whole row, or a run of at most 19456 vectors of it, then writes it: 1 - 5 %
 *                      faster); 0: one 256-lane workgroup per row.  The same bits either way.
 *   "lm_head_compact"  1 (default): fopd_lm_head_token_logprobs projects only the rows with mask != 0;
 *                      fopd_lm_head_loss_fwd_bwd and fopd_lm_head_loss_fwd_bwd_topk_teacher move each
 *                      chunk's rows with mask != 0 to the front and leave the others out of the three contractions,
 *                      and the rows without a gradient (c_t = 0: samples of weight 0) out of the two gradient
 *                      ones (the counts stay on the device: no synchronisation); 0: every row of a chunk goes
 *                      through all three.  Per-row outputs and dhidden are the same bit for bit, dweight up to
 *                      the order of its fp32 sum over rows.
 * Returns FOPD_EINVAL for an unknown name or a value outside the stated set.
 */
fopd_status fopd_set_option(const char* name, int value);

/*
 * The same two outputs as fopd_token_logprobs, from the last hidden states and the output projection
 * instead of stored logits: z_{t,v} = sum_k hidden[t,k] * weight[v,k] is formed tile by tile on the
 * matrix cores (bf16 inputs, fp32 accumulation) and reduced on the fly, so the [T, V] logits are never
 * written.  (pi_theta^t(y | x) of Eq. "kl-diagnostics" is the softmax of this projection; the paper's
 * students are Qwen models, App. B, whose projection is [V, d] = [151,936, 4096].)
 *
 *   hidden      [T, ldh] bf16, ldh >= d           weight      [V, ldw] bf16, ldw >= d
 *   d           hidden size, a multiple of 64; V * ldw must be below 2^31 (32-bit offsets inside the matrix); rows
 *               beyond 2^31 / ldh go through in blocks of that many, launch after launch
 *   token_ids, mask, logp, lse: as in fopd_token_logprobs (masked rows give 0, 0; they are not projected: the
 *               kernel gathers the other rows through a row map and reads their count on the device, option
 *               "lm_head_compact")
 *   workspace   fopd_lm_head_workspace_bytes(T) bytes, 256-byte aligned, initialised once with
 *               fopd_workspace_init; token ids outside [0, V) raise the same sticky flag
 *
 * The logits are not rounded to bf16 on the way, so lse differs from the stored-logits call by that
 * rounding.  lp_t uses a separate fp32 dot product for z_{t,y_t} and is clamped at 0.
 * The first call in a process sets a kernel attribute (large dynamic LDS): make one call before
 * capturing this entry point into a HIP graph.  Enqueues kernels only (no memset, no allocation).
 */
size_t fopd_lm_head_workspace_bytes(int64_t T);
fopd_status fopd_lm_head_token_logprobs(const void* hidden, int64_t ldh, const void* weight, int64_t ldw,
                                        int64_t T, int64_t V, int64_t d, const int32_t* token_ids,
                                        const uint8_t* mask, float* logp, float* lse,
                                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Loss and gradient (second loop of Algorithm 1) when the logits are the output projection of the last hidden
 * states, z_{t,v} = sum_k hidden[t,k] * weight[v,k], and no [T, V] tensor is ever allocated: the pass is carried
 * through the projection and returns the gradient with respect to the hidden states and to the projection matrix,
 *   dhidden[t, :]  = sum_v dL/dz[t, v] * weight[v, :],     dweight[v, :] (+)= sum_t dL/dz[t, v] * hidden[t, :],
 * with dL/dz[t, v] = c_t (softmax(z_t)_v - [v = y_t]) exactly as in fopd_loss_fwd_bwd.
 *
 * The rows are processed in chunks of `rows_chunk`: the chunk's logits are formed on the matrix cores into
 * scratch memory (fp32, not rounded to a storage type), the log-sum-exp and gradient kernels of the stored-logits
 * path run on them (the gradient rows are written as bf16, as that path stores them), and two more matrix-core
 * contractions fold the rows into dhidden and dweight; then the scratch is reused.  All work is bf16 inputs with
 * fp32 accumulation; the result does not depend on rows_chunk except through the order of the fp32 sums over
 * rows in dweight.  Rows with mask == 0 (observations, prompts: no log-prob, no gradient row) cost no matrix work:
 * each chunk's other rows are gathered to the front, the kernels run on those, and the per-row outputs and dhidden
 * rows are scattered back, zeros at the masked rows; likewise the rows of samples of weight 0 are left out of the
 * two gradient contractions (option "lm_head_compact").
 *
 * Scores, two ways:
 *   freshness_in != NULL  [B] f32 scores formed earlier (Algorithm 1 scores the buffer before its minibatch loop;
 *                         with no logits kept, fopd_lm_head_token_logprobs followed by fopd_freshness_score gives
 *                         them from the same inputs); n_train_in / n_roll_in [B] int32 from fopd_freshness_score,
 *                         or NULL to count from `mask`.  Chunks are rows_chunk rows each and may cut samples.
 *   freshness_in == NULL  the scores are formed inside the call from the chunk's own log-probs, as
 *                         fopd_loss_fwd_bwd does when it is given none: the projection is then computed once per
 *                         step, not twice.  Chunks gather whole samples (as many as fit into rows_chunk rows), so
 *                         the host must know the lengths: seq_lens_host [B] int32 (HOST memory, the same values
 *                         as seq_lens), n_train_in and n_roll_in NULL.  If a sample is longer than rows_chunk rows
 *                         the call sweeps the rows twice in chunks of rows_chunk rows instead: logits and
 *                         log-probs of every chunk first (one more contraction per chunk), then the scores of all
 *                         samples, then the pass as if they had been supplied - the same results with four
 *                         contractions per chunk instead of three.  D^sup is 0 in this mode (no stale teacher
 *                         log-probs are taken).
 *
 *   hidden [T, ldh] bf16, weight [V, ldw] bf16, d a multiple of 64; token_ids, mask, behav_logp, teacher_logp,
 *   seq_lens (sum == T), lag, B, hp, grad_scale as in fopd_loss_fwd_bwd
 *   rows_chunk   rows per chunk, a multiple of 64 (scratch at V = 151,936, d = 4096: 9.0 GB for 8192 rows, 16.7 GB for 16384, which is 4 - 10 % faster)
 *   loss [1], freshness [B] (may be NULL; a copy of freshness_in when that is given), weights [B] (may be NULL),
 *   logp [T], lse [T]: f32 outputs.  With freshness_in given (and both gradient outputs) the two may be NULL together
 *                (the caller has them from the scoring call): the samples of weight 0 are then left out of the call
 *                altogether, none of their rows is projected (needs option "lm_head_compact" = 1, the default)
 *   dhidden [T, lddh] f32 out; dweight [V, lddw] f32: overwritten, or added to when accumulate_dweight != 0.
 *                dweight NULL, dhidden given: the projection is not trained (a frozen or tied head whose gradient
 *                is formed elsewhere): two contractions per chunk instead of three.
 *                Both NULL (with freshness_in == NULL): the call only scores - log-probs, scores, weights and the
 *                loss of the first loop of Algorithm 1 on projected logits, one contraction per chunk instead of three
 *   workspace    fopd_lm_head_loss_workspace_bytes(T, V, d, B, rows_chunk) bytes, 256-byte aligned, initialised
 *                once with fopd_workspace_init; the same sticky flags as the other entry points
 * The first call in a process sets kernel attributes: make one call before capturing it into a HIP graph.
 */
size_t fopd_lm_head_loss_workspace_bytes(int64_t T, int64_t V, int64_t d, int32_t B, int64_t rows_chunk);
fopd_status fopd_lm_head_loss_fwd_bwd(const void* hidden, int64_t ldh, const void* weight, int64_t ldw, int64_t T,
                                      int64_t V, int64_t d, const int32_t* token_ids, const uint8_t* mask,
                                      const float* behav_logp, const float* teacher_logp, const int32_t* seq_lens,
                                      const int32_t* lag, int32_t B, fopd_hparams hp, const float* freshness_in,
                                      const int32_t* n_train_in, const int32_t* n_roll_in,
                                      const int32_t* seq_lens_host, float grad_scale, int64_t rows_chunk,
                                      float* loss, float* freshness, float* weights, float* logp, float* lse,
                                      float* dhidden, int64_t lddh, float* dweight, int64_t lddw,
                                      int accumulate_dweight, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same pass through the projection with the distribution-level token loss against a teacher stored as k tokens
 * per row (the loss, coarsening and gradient of fopd_loss_fwd_bwd_topk_teacher, on logits that exist only chunk by
 * chunk): per chunk of whole samples the logits are formed in fp32 scratch, the log-sum-exp kernel and the listed
 * terms run on them, the samples' scores follow at once (the freshness_in == NULL mode of
 * fopd_lm_head_loss_fwd_bwd: one projection per step), the gradient rows are written as bf16 with one coefficient
 * per row and corrected at the k listed tokens and the sampled one, and the two contractions fold them into dhidden
 * and dweight.
 *   list_ids, list_logp [T, k], k, rest_floor     as in fopd_loss_fwd_bwd_topk_teacher
 *   teacher_logp, teacher_logp_stale [T] or NULL  the sampled token's teacher log-probabilities, for D^sup only
 *                                                 (D^sup = 0 unless both are given; the stale one alone is FOPD_EINVAL)
 *   freshness_in, n_train_in, n_roll_in           NULL: the scores are formed inside the call, as described above
 *                                                 (seq_lens_host is then needed).  Given: scores formed earlier
 *                                                 (the scoring-only form of this call over the buffer gives them),
 *                                                 exactly as in fopd_lm_head_loss_fwd_bwd: chunks may cut samples,
 *                                                 seq_lens_host is not read, both gradient outputs are required
 *   seq_lens_host [B] int32 (HOST memory, the values of seq_lens); with a sample longer than rows_chunk rows the
 *                                                 call sweeps the rows twice, as fopd_lm_head_loss_fwd_bwd does
 *   token_loss [T] f32 out or NULL (l_t; 0 outside U^sup); the other arguments as in fopd_lm_head_loss_fwd_bwd,
 *   dhidden and dweight both NULL included (scoring only: the buffer's listed-teacher scores without a gradient pass)
 *   workspace  fopd_lm_head_loss_topk_workspace_bytes(T, V, d, B, rows_chunk, k) bytes
 */
size_t fopd_lm_head_loss_topk_workspace_bytes(int64_t T, int64_t V, int64_t d, int32_t B, int64_t rows_chunk,
                                              int32_t k);
fopd_status fopd_lm_head_loss_fwd_bwd_topk_teacher(
    const void* hidden, int64_t ldh, const void* weight, int64_t ldw, int64_t T, int64_t V, int64_t d,
    const int32_t* token_ids, const uint8_t* mask, const float* behav_logp, const int32_t* list_ids,
    const float* list_logp, int32_t k, float rest_floor, const float* teacher_logp, const float* teacher_logp_stale,
    const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp, const float* freshness_in,
    const int32_t* n_train_in, const int32_t* n_roll_in, const int32_t* seq_lens_host, float grad_scale,
    int64_t rows_chunk, float* loss, float* freshness, float* weights, float* logp, float* lse, float* token_loss,
    float* dhidden, int64_t lddh, float* dweight, int64_t lddw, int accumulate_dweight, void* workspace,
    size_t workspace_bytes, void* stream);

/*
 * Per-kernel timing for benchmarks.  While enabled, every launch of the two streaming kernels
 * is bracketed by HIP events on the launch stream (process-wide state behind the library's mutex; the
 * events are created on first use, so do not enable it around code that may not allocate).
 * fopd_profile_read is HOST-SYNCHRONOUS (waits for the recorded events).
 *   which: 0 = log-sum-exp pass, 1 = gradient pass, 2 = both passes in one kernel (scores supplied),
 *          3 = projection fused with the log-sum-exp; of fopd_lm_head_loss_fwd_bwd: 4 = logits contraction,
 *          5 = dhidden contraction, 6 = dweight contraction.
 */
fopd_status fopd_profile_enable(int on);
fopd_status fopd_profile_reset(void);
fopd_status fopd_profile_read(int which, double* total_ms_host, int64_t* launches_host);

#ifdef __cplusplus
}
#endif
#endif /* FOPD_H */
