// Host side of the C ABI declared in include/fopd.h: argument checks, workspace carving and
// kernel launches.  Nothing here allocates device memory or synchronises, apart from the
// two documented host-synchronous helpers.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <string>
#include <vector>

#include "fopd.h"
#include "fopd_kernels.hip"
#include "fopd_lm_head.hip"
#include "fopd_gemm.hip"

namespace {

using namespace fopd;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Carving of the caller's workspace.  Every region starts on a 256-byte boundary.
struct Workspace {
  size_t flags = 0, cu = 0, n_train = 0, n_roll = 0, fresh64 = 0, coef = 0, lse = 0, logp = 0, coef2 = 0, dlse = 0,
         kl = 0, logq = 0, partials = 0, total = 0;
  static constexpr size_t take(size_t& off, size_t bytes) {
    const size_t at = off;
    off = (off + bytes + 255) / 256 * 256;
    return at;
  }
  constexpr Workspace(int64_t T, int32_t B) {
    const size_t t = static_cast<size_t>(T < 0 ? 0 : T), b = static_cast<size_t>(B < 0 ? 0 : B);
    size_t off = 0;
    flags = take(off, 4 * sizeof(int32_t));
    cu = take(off, (b + 1) * sizeof(int64_t));
    n_train = take(off, b * sizeof(int32_t));
    n_roll = take(off, b * sizeof(int32_t));
    fresh64 = take(off, b * sizeof(double));
    coef = take(off, t * sizeof(float));
    lse = take(off, t * sizeof(float));
    logp = take(off, t * sizeof(float));
    coef2 = take(off, t * sizeof(float));
    dlse = take(off, t * sizeof(float));
    kl = take(off, t * sizeof(float));
    logq = take(off, t * sizeof(float));
    partials = take(off, (t + 1) * sizeof(double));     // per-block or per-row loss terms
    total = off;
  }
};

// Workspace of the projection-fused log-prob call: the same flag words, then one (reference, sum) pair per
// strip and token, the tokens padded to whole tiles.
struct LmWorkspace {
  size_t flags, n_live, partial, ex, row_map, t_pad, total;
  explicit LmWorkspace(int64_t T) {
    const size_t t = static_cast<size_t>(T < 0 ? 0 : T);
    t_pad = (t + kLmTile - 1) / kLmTile * kLmTile;
    flags = 0;
    n_live = 128;                                        // the count of unmasked rows, on the device
    partial = 256;
    ex = align_up(partial + static_cast<size_t>(kLmStripsMax) * t_pad * sizeof(float2), 256);
    row_map = align_up(ex + (t + 1) * sizeof(int32_t), 256);
    total = align_up(row_map + t * sizeof(int32_t), 256);
  }
};

// ---- scratch memory owned by the library, for the entry point that may not allocate -------------------
// One workspace of the largest size that entry point accepts, as a device array of this module: every GPU the
// library runs on holds its own copy from module load until the process ends.
constexpr int64_t kStaticMaxRows = FOPD_STATIC_MAX_ROWS;
constexpr int32_t kStaticMaxSamples = FOPD_STATIC_MAX_SAMPLES;
constexpr size_t kStaticBytes = Workspace(kStaticMaxRows, kStaticMaxSamples).total;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

// In host code `scratch` is only a handle for the runtime: the array's device address is looked up once per
// device (with that device current) and kept; host code uses that address, never the symbol's name.
void* g_scratch_ptr[64] = {};

// Workspace of the loss pass through the projection: flags, offsets and counts, the per-chunk O(R) arrays, then
// the chunk's fp32 logits, its bf16 gradient rows and the transposed projection matrix.  ldz = V rounded up to 64
// (the k-extent of the dL/dhidden contraction).
struct LmLossWorkspace {
  size_t flags = 0, cu = 0, n_train = 0, n_roll = 0, fresh64 = 0, coef = 0, partials = 0, chunk_loss = 0, z = 0, g = 0,
         wt = 0, total = 0;
  // with a teacher stored as k tokens per row: token loss [T], per-row values and per-slot terms of one chunk
  size_t token_loss = 0, c2 = 0, g_rest = 0, row_coef = 0, p_list = 0, h_list = 0;
  // the chunk's live rows moved to the front: prefix counts, row map, live count, sample offsets, then the dense
  // copies of the per-row inputs and outputs, of the hidden rows and of their gradient
  // and, for the gradient side, the same among the live rows for those that have a gradient row
  size_t ex = 0, row_map = 0, n_live = 0, cu_c = 0, tok_c = 0, mask_c = 0, behav_c = 0, teach_c = 0, stale_c = 0,
         logp_c = 0, lse_c = 0, tl_c = 0, ids_c = 0, llp_c = 0, h_c = 0, dh_c = 0, grad_ex = 0, h_g = 0, keep = 0;
  int64_t ldz = 0, r_pad = 0, n_chunks = 0;
  LmLossWorkspace(int64_t T, int64_t V, int64_t d, int32_t B, int64_t rows_chunk, int32_t k = 0) {
    const size_t b = static_cast<size_t>(B < 0 ? 0 : B);
    const int64_t t = T < 0 ? 0 : T;
    const int64_t rc = rows_chunk < 64 ? 64 : rows_chunk;
    const size_t r = static_cast<size_t>(t < rc ? (t + 63) / 64 * 64 : rc);     // rows of the largest chunk, padded
    r_pad = static_cast<int64_t>(r);
    n_chunks = (t + rc - 1) / rc;
    ldz = (V + 63) / 64 * 64;
    const size_t dd = static_cast<size_t>(d < 0 ? 0 : d);
    size_t off = 0;
    flags = Workspace::take(off, 4 * sizeof(int32_t));
    cu = Workspace::take(off, (b + 1) * sizeof(int64_t));
    n_train = Workspace::take(off, b * sizeof(int32_t));
    n_roll = Workspace::take(off, b * sizeof(int32_t));
    fresh64 = Workspace::take(off, b * sizeof(double));
    coef = Workspace::take(off, r * sizeof(float));
    partials = Workspace::take(off, (r / kStreamThreads + 2) * sizeof(double));
    // chunks that follow sample boundaries (scores formed inside the call) are at most n_chunks + B
    chunk_loss = Workspace::take(off, (static_cast<size_t>(n_chunks) + b + 1) * sizeof(float));
    z = Workspace::take(off, r * static_cast<size_t>(ldz) * sizeof(float));
    g = Workspace::take(off, r * static_cast<size_t>(ldz) * 2);
    wt = Workspace::take(off, dd * static_cast<size_t>(ldz) * 2);
    if (k > 0) {
      const size_t kk = static_cast<size_t>(k);
      token_loss = Workspace::take(off, static_cast<size_t>(t) * sizeof(float));
      c2 = Workspace::take(off, r * sizeof(float));
      g_rest = Workspace::take(off, r * sizeof(float));
      row_coef = Workspace::take(off, r * sizeof(float));
      p_list = Workspace::take(off, r * kk * sizeof(float));
      h_list = Workspace::take(off, r * kk * sizeof(float));
      ids_c = Workspace::take(off, r * kk * sizeof(int32_t));
      llp_c = Workspace::take(off, r * kk * sizeof(float));
    }
    ex = Workspace::take(off, (static_cast<size_t>(t) + 1) * sizeof(int32_t));     // (a whole call's rows when the
    row_map = Workspace::take(off, static_cast<size_t>(t) * sizeof(int32_t));       //  scores are supplied)
    n_live = Workspace::take(off, 64 * sizeof(int32_t));
    cu_c = Workspace::take(off, (b + 1) * sizeof(int64_t));
    tok_c = Workspace::take(off, r * sizeof(int32_t));
    mask_c = Workspace::take(off, r);
    behav_c = Workspace::take(off, r * sizeof(float));
    teach_c = Workspace::take(off, r * sizeof(float));
    stale_c = Workspace::take(off, r * sizeof(float));
    logp_c = Workspace::take(off, r * sizeof(float));
    lse_c = Workspace::take(off, r * sizeof(float));
    tl_c = Workspace::take(off, r * sizeof(float));
    h_c = Workspace::take(off, r * dd * 2);
    dh_c = Workspace::take(off, r * dd * sizeof(float));
    grad_ex = Workspace::take(off, (r + 1) * sizeof(int32_t));
    h_g = Workspace::take(off, r * dd * 2);
    keep = Workspace::take(off, b * sizeof(int32_t));
    total = off;
  }
};

// The teacher of the loss pass through the projection when it is stored as k tokens per row.
struct ListedTeacher {
  const int32_t* ids = nullptr;
  const float* logp = nullptr;
  int32_t k = 0;
  float rest_floor = 0.f;
  const float* teacher_logp_stale = nullptr;     // with teacher_logp: the sampled token's, for D^sup
  float* token_loss = nullptr;                   // [T] out, may be NULL
};

template <typename P>
inline P* at(void* ws, size_t off) {
  return reinterpret_cast<P*>(static_cast<char*>(ws) + off);
}

inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

fopd_status check_matrix(const void* m, fopd_dtype dt, int64_t T, int64_t V, int64_t ld) {
  if (dt != FOPD_F32 && dt != FOPD_BF16) return FOPD_EDTYPE;
  if (T < 0 || T > 2147483647LL || V <= 0 || ld < V || V > 2147483647LL - 16) return FOPD_ESHAPE;
  if (m == nullptr) return FOPD_EINVAL;
  const size_t es = (dt == FOPD_F32) ? 4 : 2;
  if (misaligned(m, 16) || (static_cast<size_t>(ld) * es) % 16 != 0) return FOPD_EALIGN;
  return FOPD_OK;
}

fopd_status check_workspace(const void* ws, size_t bytes, int64_t T, int32_t B) {
  if (ws == nullptr || misaligned(ws, 256)) return FOPD_EWORKSPACE;
  if (bytes < Workspace(T, B).total) return FOPD_EWORKSPACE;
  return FOPD_OK;
}

inline fopd_status launched() { return hipGetLastError() == hipSuccess ? FOPD_OK : FOPD_EHIP; }

// ---- the library's only process-wide state: launch-shape options, the optional timing events and the
// per-device "attribute already set" tables.  All of it sits behind one mutex; the entry points hold it
// only while they read or update this state, never across a launch.
std::mutex g_state_mutex;

// ---- optional per-kernel timing ---------------------------------------------------------
constexpr int kProfSlots = 8;
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> start[kProfSlots], stop[kProfSlots];
  size_t used[kProfSlots] = {};
} g_prof;

// Brackets the launches made during its lifetime with a pair of events when timing is switched on.
// `allowed` = false (the entry point that may not allocate: event creation allocates) records nothing.
struct ScopedTimer {
  hipEvent_t stop = nullptr;
  hipStream_t s;
  ScopedTimer(int w, hipStream_t st, bool allowed = true) : s(st) {
    if (!allowed) return;
    hipEvent_t start = nullptr;
    {
      std::lock_guard<std::mutex> lock(g_state_mutex);
      if (!g_prof.on) return;
      if (g_prof.used[w] == g_prof.start[w].size()) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
        g_prof.start[w].push_back(a);
        g_prof.stop[w].push_back(b);
      }
      const size_t slot = g_prof.used[w]++;
      start = g_prof.start[w][slot];
      stop = g_prof.stop[w][slot];
    }
    (void)hipEventRecord(start, s);
  }
  ~ScopedTimer() {
    if (stop != nullptr) (void)hipEventRecord(stop, s);
  }
};

// ---- options ------------------------------------------------------------------------------
struct Options {
  int k14_threads = 256;          // lanes per row in the two-pass-per-row kernel
  int k14_rows_per_cu = 6;        // rows in flight per compute unit (measured optimum on MI355X)
  int k14_regs_grid = 0;          // workgroups of the row-in-registers kernel; 0 = two per compute unit
  int k14_regs = 1;               // 1: rows that fit (16-byte vectors <= 1024 x 19) are held in registers between the passes
  int lm_head_compact = 1;        // 1: the loss pass through the projection leaves masked rows out of its contractions
  int k4_regs = 1;                // 1: the gradient kernel holds a row in registers between its loads and stores
} g_opt;

inline Options current_options() {
  std::lock_guard<std::mutex> lock(g_state_mutex);
  return g_opt;
}

constexpr size_t kLdsPerCu = 160 * 1024;

// A kernel that wants more dynamic LDS than the default limit has to be told so once per device.
// `done` is the caller's per-kernel table of devices already told.
constexpr int kMaxDevices = 64;
inline fopd_status allow_dynamic_lds(const void* kern, int bytes, bool* done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FOPD_EHIP;
  std::lock_guard<std::mutex> lock(g_state_mutex);
  if (done[dev]) return FOPD_OK;
  if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return FOPD_EHIP;
  done[dev] = true;
  return FOPD_OK;
}

// Compute units of the current device (256 when the runtime cannot say).
inline int compute_units() {
  static int cached[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  std::lock_guard<std::mutex> lock(g_state_mutex);
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
      (void)hipGetLastError();
      n = 256;
    }
    cached[dev] = n;
  }
  return cached[dev];
}

// Device address of `scratch` on the current device.
inline fopd_status static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FOPD_EHIP;
  std::lock_guard<std::mutex> lock(g_state_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return FOPD_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return FOPD_OK;
}

// ---- launch helpers ---------------------------------------------------------------------

fopd_status launch_k1(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                      const int32_t* token_ids, const uint8_t* mask, float* logp, float* lse,
                      int64_t* gather_idx, float* entropy, int32_t* flags, hipStream_t s, bool timed = true) {
  if (T == 0) return FOPD_OK;
  ScopedTimer timer(0, s, timed);
  const dim3 grid(static_cast<unsigned>(T)), block(kStreamThreads);
  const int v = static_cast<int>(V);
#define FOPD_K1_ARGS logits, T, v, ld, token_ids, mask, logp, lse, gather_idx, entropy, flags
  if (dt == FOPD_BF16) {
    if (entropy != nullptr) fopd_k1_lse<FOPD_BF16, kUnroll, true><<<grid, block, 0, s>>>(FOPD_K1_ARGS);
    else fopd_k1_lse<FOPD_BF16, kUnroll, false><<<grid, block, 0, s>>>(FOPD_K1_ARGS);
  } else {
    if (entropy != nullptr) fopd_k1_lse<FOPD_F32, kUnroll, true><<<grid, block, 0, s>>>(FOPD_K1_ARGS);
    else fopd_k1_lse<FOPD_F32, kUnroll, false><<<grid, block, 0, s>>>(FOPD_K1_ARGS);
  }
#undef FOPD_K1_ARGS
  return launched();
}

fopd_status launch_k4(const void* logits, void* dlogits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                      const int32_t* token_ids, const float* lse, const float* logp, const float* coef,
                      hipStream_t s, bool timed = true) {
  if (T == 0) return FOPD_OK;
  const Options opt = current_options();
  ScopedTimer timer(1, s, timed);
  constexpr int kRegRowVectors = 19;
  const int64_t nvec = V / (dt == FOPD_BF16 ? 8 : 4);
  if (opt.k4_regs != 0 && nvec > 2 * 1024) {
    // the row-in-registers shape: workgroups of 1024 lanes, one resident per compute unit at a time; a row longer
    // than 1024 x 19 vectors goes in equal runs of at most that many
    const int64_t per = 1024LL * kRegRowVectors;
    const int segments = static_cast<int>((nvec + per - 1) / per);
    const int seg_vecs = static_cast<int>((nvec + segments - 1) / segments);
    // (sixteen workgroups per compute unit, handed out as the units finish: 1 % faster than two where the placement
    // of the buffers makes some units slower than others, the same elsewhere)
    const int64_t wgs = 16 * compute_units(), items = T * segments;
    const dim3 grid(static_cast<unsigned>(items < wgs ? items : wgs)), block(1024);
    if (dt == FOPD_BF16)
      fopd_k4_grad_regs<FOPD_BF16, kRegRowVectors><<<grid, block, 0, s>>>(
          logits, dlogits, T, static_cast<int>(V), ld, token_ids, lse, logp, coef, segments, seg_vecs);
    else
      fopd_k4_grad_regs<FOPD_F32, kRegRowVectors><<<grid, block, 0, s>>>(
          logits, dlogits, T, static_cast<int>(V), ld, token_ids, lse, logp, coef, segments, seg_vecs);
    return launched();
  }
  const dim3 grid(static_cast<unsigned>(T)), block(kGradThreads);
  if (dt == FOPD_BF16)
    fopd_k4_grad<FOPD_BF16, kGradUnroll><<<grid, block, 0, s>>>(logits, dlogits, T, static_cast<int>(V), ld,
                                                            token_ids, lse, logp, coef);
  else
    fopd_k4_grad<FOPD_F32, kGradUnroll><<<grid, block, 0, s>>>(logits, dlogits, T, static_cast<int>(V), ld,
                                                           token_ids, lse, logp, coef);
  return launched();
}

// Everything the two-passes-per-row kernel needs besides the matrices.
struct RowPassArgs {
  const int32_t* token_ids;
  const uint8_t* mask;
  const float* lb;
  const float* lq;
  const int64_t* cu;
  const int32_t* n_train;
  const int32_t* n_roll;
  const int32_t* lag;
  const float* fresh32;
  int32_t B;
  int64_t row_begin;
  fopd_hparams hp;
  float grad_scale;
  float* logp;
  double* row_loss;
  int32_t* flags;
};

template <int DT, int NT>
fopd_status launch_k14_t(const void* logits, void* dlogits, int64_t T, int64_t V, int64_t ld, const RowPassArgs& a,
                         int rows_per_cu, hipStream_t s) {
  auto kern = fopd_k14_fused<DT, NT, kUnroll>;
  // dynamic LDS is requested only to cap the workgroups resident per compute unit; the kernel is told
  // once per instantiation and device that it may be given up to a whole CU's worth
  static bool allowed[kMaxDevices] = {};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), static_cast<int>(kLdsPerCu - 1024), allowed) != FOPD_OK)
    return FOPD_EHIP;
  const size_t pad = kLdsPerCu / static_cast<size_t>(rows_per_cu) - 1024;
  kern<<<dim3(static_cast<unsigned>(T)), dim3(NT), pad, s>>>(logits, dlogits, T, static_cast<int>(V), ld, a.token_ids,
                                                            a.mask, a.lb, a.lq, a.cu, a.n_train, a.n_roll, a.lag,
                                                            a.fresh32, a.B, a.row_begin, a.hp, a.grad_scale, a.logp,
                                                            a.row_loss, a.flags);
  return launched();
}

fopd_status launch_k14(const void* logits, void* dlogits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                       const RowPassArgs& a, hipStream_t s, bool timed) {
  if (T == 0) return FOPD_OK;
  const Options opt = current_options();
  ScopedTimer timer(2, s, timed);
  constexpr int kRegRowVectors = 19;
  const int64_t nvec = V / (dt == FOPD_BF16 ? 8 : 4);
  if (opt.k14_regs != 0 && nvec <= static_cast<int64_t>(kRegRowThreads) * kRegRowVectors && nvec > 2 * kRegRowThreads) {
    // One workgroup is resident per compute unit (it takes the whole register file) and walks rows in steps of the
    // grid.  Twice as many workgroups as compute units: the second half is handed out as compute units finish, which
    // evens out their unequal speeds (measured: as fast as one per compute unit when all run alike, 4 % faster when
    // the placement of the two buffers makes some slower).
    const int64_t cus = (opt.k14_regs_grid > 0) ? opt.k14_regs_grid : 2 * compute_units();
    const dim3 grid(static_cast<unsigned>(T < cus ? T : cus)), block(kRegRowThreads);
    if (dt == FOPD_BF16)
      fopd_k14_regs<FOPD_BF16, kRegRowVectors><<<grid, block, 0, s>>>(
          logits, dlogits, T, static_cast<int>(V), ld, a.token_ids, a.mask, a.lb, a.lq, a.cu, a.n_train, a.n_roll, a.lag,
          a.fresh32, a.B, a.row_begin, a.hp, a.grad_scale, a.logp, a.row_loss, a.flags);
    else
      fopd_k14_regs<FOPD_F32, kRegRowVectors><<<grid, block, 0, s>>>(
          logits, dlogits, T, static_cast<int>(V), ld, a.token_ids, a.mask, a.lb, a.lq, a.cu, a.n_train, a.n_roll, a.lag,
          a.fresh32, a.B, a.row_begin, a.hp, a.grad_scale, a.logp, a.row_loss, a.flags);
    return launched();
  }
#define FOPD_K14_CASE(DTV, NTV) return launch_k14_t<DTV, NTV>(logits, dlogits, T, V, ld, a, opt.k14_rows_per_cu, s)
  if (dt == FOPD_BF16) {
    if (opt.k14_threads == 512) FOPD_K14_CASE(FOPD_BF16, 512);
    if (opt.k14_threads == 1024) FOPD_K14_CASE(FOPD_BF16, 1024);
    FOPD_K14_CASE(FOPD_BF16, 256);
  }
  if (opt.k14_threads == 512) FOPD_K14_CASE(FOPD_F32, 512);
  if (opt.k14_threads == 1024) FOPD_K14_CASE(FOPD_F32, 1024);
  FOPD_K14_CASE(FOPD_F32, 256);
#undef FOPD_K14_CASE
}

// The body of fopd_loss_fwd_bwd once its arguments have been checked.  `timed` = false keeps the optional
// timing events (whose creation allocates) out of the call.
fopd_status loss_fwd_bwd_checked(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                 const int32_t* token_ids, const uint8_t* mask, const float* behav_logp,
                                 const float* teacher_logp, const float* teacher_logp_stale,
                                 const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp,
                                 const float* freshness_in, const int32_t* n_train_in, const int32_t* n_roll_in,
                                 int64_t row_begin, const float* lse_in, const float* logp_in, float grad_scale,
                                 float* loss, float* freshness, float* weights, float* logp, void* dlogits,
                                 void* workspace, hipStream_t s, bool timed) {
  const bool scored = (freshness_in != nullptr);
  const bool have_lse = (lse_in != nullptr);
  fopd_status st;
  const Workspace w(T, B);
  int32_t* flags = at<int32_t>(workspace, w.flags);
  int64_t* cu = at<int64_t>(workspace, w.cu);
  int32_t* nws = at<int32_t>(workspace, w.n_train);
  int32_t* nrws = at<int32_t>(workspace, w.n_roll);
  double* f64 = at<double>(workspace, w.fresh64);
  float* coef = at<float>(workspace, w.coef);
  float* lse_ws = at<float>(workspace, w.lse);
  float* logp_ws = (logp != nullptr) ? logp : at<float>(workspace, w.logp);
  double* partials = at<double>(workspace, w.partials);

  // segment offsets; whole-sample calls must cover exactly T rows, chunks at least their range
  const bool whole = (n_train_in == nullptr);
  fopd_scan_seqlens<<<1, kScanThreads, 0, s>>>(seq_lens, lag, B, whole ? T : -1, row_begin + T, cu, flags);
  if ((st = launched()) != FOPD_OK) return st;

  // Scores supplied, log-probs not: both passes over each row run in one kernel, and the second
  // read of the row comes out of the cache.
  if (scored && !have_lse) {
    const int32_t* n_use = n_train_in;
    const int32_t* nr_use = n_roll_in;                  // NULL: the two counts coincide
    if (whole) {
      fopd_count_train<<<B, kSegThreads, 0, s>>>(mask, cu, T, nws, nrws);
      if ((st = launched()) != FOPD_OK) return st;
      n_use = nws;
      nr_use = nrws;
    }
    const RowPassArgs a{token_ids, mask, behav_logp, teacher_logp, cu, n_use, nr_use, lag, freshness_in, B,
                        row_begin, hp, grad_scale, logp, partials, flags};
    if ((st = launch_k14(logits, dlogits, dt, T, V, ld, a, s, timed)) != FOPD_OK) return st;
    fopd_loss_final<<<1, kSegThreads, 0, s>>>(partials, T, n_use, nr_use, lag, nullptr, freshness_in, B, hp.xi, loss,
                                              weights, freshness);
    return launched();
  }

  // token log-probabilities: computed here, or taken from an earlier fopd_token_logprobs
  const float* lse_use = lse_in;
  const float* logp_use = logp_in;
  if (!have_lse) {
    st = launch_k1(logits, dt, T, V, ld, token_ids, mask, logp_ws, lse_ws, nullptr, nullptr, flags, s, timed);
    if (st != FOPD_OK) return st;
    lse_use = lse_ws;
    logp_use = logp_ws;
  } else if (logp != nullptr && logp != logp_in && T > 0) {
    if (hipMemcpyAsync(logp, logp_in, static_cast<size_t>(T) * sizeof(float), hipMemcpyDeviceToDevice, s) !=
        hipSuccess)
      return FOPD_EHIP;
  }

  // per-sample counts and scores
  const int32_t* n_use = n_train_in;
  const int32_t* nr_use = n_roll_in;                    // NULL: the two counts coincide
  if (whole) {
    fopd_segment_stats<<<B, kSegThreads, 0, s>>>(logp_use, behav_logp, nullptr, nullptr, teacher_logp, teacher_logp_stale,
                                                 mask, cu, lag, T, hp, nullptr, nullptr, nullptr, nullptr, nullptr,
                                                 nullptr, nullptr, nullptr, f64, nws, nrws);
    if ((st = launched()) != FOPD_OK) return st;
    n_use = nws;
    nr_use = nrws;
  }
  const double* f64_use = scored ? nullptr : f64;

  const int64_t nblk = (T + kStreamThreads - 1) / kStreamThreads;
  if (T > 0) {
    fopd_coef_loss<<<static_cast<unsigned>(nblk), kStreamThreads, 0, s>>>(
        logp_use, behav_logp, teacher_logp, mask, cu, n_use, nr_use, lag, f64_use, freshness_in, T, B, row_begin, hp,
        grad_scale, coef, partials, flags);
    if ((st = launched()) != FOPD_OK) return st;
  }
  fopd_loss_final<<<1, kSegThreads, 0, s>>>(partials, nblk, n_use, nr_use, lag, f64_use, freshness_in, B, hp.xi, loss,
                                            weights, freshness);
  if ((st = launched()) != FOPD_OK) return st;

  return launch_k4(logits, dlogits, dt, T, V, ld, token_ids, lse_use, logp_use, coef, s, timed);
}

// Host-checkable conditions of fopd_loss_fwd_bwd other than the workspace.
fopd_status loss_fwd_bwd_check_args(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                    const int32_t* token_ids, const float* behav_logp, const float* teacher_logp,
                                    const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp,
                                    const float* freshness_in, const int32_t* n_train_in, const int32_t* n_roll_in,
                                    int64_t row_begin, const float* lse_in, const float* logp_in, const float* loss,
                                    const void* dlogits) {
  fopd_status st = check_matrix(logits, dt, T, V, ld);
  if (st != FOPD_OK) return st;
  if ((st = check_matrix(dlogits, dt, T, V, ld)) != FOPD_OK) return st;
  if (B <= 0 || row_begin < 0) return FOPD_ESHAPE;
  if (token_ids == nullptr || behav_logp == nullptr || teacher_logp == nullptr || seq_lens == nullptr ||
      lag == nullptr || loss == nullptr)
    return FOPD_EINVAL;
  if (!(hp.alpha >= 0.f) || !(hp.beta >= 0.f)) return FOPD_EINVAL;
  const bool scored = (freshness_in != nullptr);
  const bool have_lse = (lse_in != nullptr);
  if (have_lse != (logp_in != nullptr)) return FOPD_EINVAL;
  if (!scored && (have_lse || n_train_in != nullptr || row_begin != 0)) return FOPD_EINVAL;
  if (n_roll_in != nullptr && n_train_in == nullptr) return FOPD_EINVAL;
  if (scored && n_train_in == nullptr && row_begin != 0) return FOPD_EINVAL;
  return FOPD_OK;
}

}  // namespace

extern "C" {

const char* fopd_status_string(fopd_status status) {
  switch (status) {
    case FOPD_OK: return "ok";
    case FOPD_EINVAL: return "invalid argument (NULL pointer, negative coefficient or inconsistent optional inputs)";
    case FOPD_ESHAPE: return "invalid shape (T, V, B, ld)";
    case FOPD_EALIGN: return "matrix base or row pitch is not 16-byte aligned";
    case FOPD_EDTYPE: return "unsupported element type";
    case FOPD_EWORKSPACE: return "workspace missing, misaligned or too small";
    case FOPD_ETOKEN_RANGE: return "token id outside [0, V) (row treated as masked)";
    case FOPD_ESEGMENTS: return "sequence lengths negative or not covering the rows of the call";
    case FOPD_ELAG: return "negative lag (sample treated as invalid)";
    case FOPD_EHIP: return "HIP runtime or launch failure";
    case FOPD_ESETS: return "mask names two different aligned sets but only one count array was given (rows dropped)";
    case FOPD_ELIMIT: return "size beyond the fixed limits of the entry point";
    default: return "unknown status";
  }
}

size_t fopd_workspace_bytes(int64_t T, int32_t B) { return Workspace(T, B).total; }

fopd_status fopd_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (workspace == nullptr || misaligned(workspace, 256) || workspace_bytes < 256) return FOPD_EWORKSPACE;
  fopd_clear_flags<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>(static_cast<int32_t*>(workspace));
  return launched();
}

fopd_status fopd_workspace_status(const void* workspace, void* stream, int32_t* flags_host) {
  if (workspace == nullptr) return FOPD_EWORKSPACE;
  int32_t f = 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&f, workspace, sizeof(f), hipMemcpyDeviceToHost, s) != hipSuccess) return FOPD_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return FOPD_EHIP;
  if (flags_host != nullptr) *flags_host = f;
  return fopd_flags_status(f);
}

fopd_status fopd_flags_status(int32_t flags) {
  if (flags & kFlagToken) return FOPD_ETOKEN_RANGE;
  if (flags & kFlagSegments) return FOPD_ESEGMENTS;
  if (flags & kFlagLag) return FOPD_ELAG;
  if (flags & kFlagSets) return FOPD_ESETS;
  return FOPD_OK;
}

fopd_status fopd_token_logprobs(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                const int32_t* token_ids, const uint8_t* mask, float* logp, float* lse,
                                int64_t* gather_idx, float* entropy, void* workspace, size_t workspace_bytes,
                                void* stream) {
  fopd_status st = check_matrix(logits, dt, T, V, ld);
  if (st != FOPD_OK) return st;
  if (token_ids == nullptr || logp == nullptr || lse == nullptr) return FOPD_EINVAL;
  st = check_workspace(workspace, workspace_bytes, T, 0);
  if (st != FOPD_OK) return st;
  Workspace w(T, 0);
  return launch_k1(logits, dt, T, V, ld, token_ids, mask, logp, lse, gather_idx, entropy,
                   at<int32_t>(workspace, w.flags), static_cast<hipStream_t>(stream));
}

fopd_status fopd_freshness_score(const float* logp, const float* behav_logp, const float* roll_kl,
                                 const float* token_loss, const float* teacher_logp,
                                 const float* teacher_logp_stale, const uint8_t* mask,
                                 const int32_t* seq_lens, const int32_t* lag, int64_t T, int32_t B,
                                 fopd_hparams hp, int64_t* cu_seqlens, int32_t* n_train, int32_t* n_roll,
                                 float* D_roll, float* D_sup, float* ell, float* cover, float* cover_roll,
                                 float* freshness, float* agg, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  if (T < 0 || B <= 0) return FOPD_ESHAPE;
  if (logp == nullptr || (behav_logp == nullptr && roll_kl == nullptr) || seq_lens == nullptr || lag == nullptr ||
      freshness == nullptr)
    return FOPD_EINVAL;
  // the sampled token's teacher log-prob is needed for the sampled-token loss and for D^sup
  if (teacher_logp == nullptr && (token_loss == nullptr || teacher_logp_stale != nullptr)) return FOPD_EINVAL;
  if (!(hp.alpha >= 0.f) || !(hp.beta >= 0.f)) return FOPD_EINVAL;
  fopd_status st = check_workspace(workspace, workspace_bytes, T, B);
  if (st != FOPD_OK) return st;
  Workspace w(T, B);
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* flags = at<int32_t>(workspace, w.flags);
  int64_t* cu = (cu_seqlens != nullptr) ? cu_seqlens : at<int64_t>(workspace, w.cu);
  int32_t* nws = at<int32_t>(workspace, w.n_train);
  int32_t* nrws = at<int32_t>(workspace, w.n_roll);
  double* f64 = at<double>(workspace, w.fresh64);

  fopd_scan_seqlens<<<1, kScanThreads, 0, s>>>(seq_lens, lag, B, T, 0, cu, flags);
  if ((st = launched()) != FOPD_OK) return st;
  fopd_segment_stats<<<B, kSegThreads, 0, s>>>(logp, behav_logp, roll_kl, token_loss, teacher_logp, teacher_logp_stale,
                                               mask, cu, lag, T, hp, n_train, n_roll, D_roll, D_sup, ell, cover,
                                               cover_roll, freshness, f64, nws, nrws);
  if ((st = launched()) != FOPD_OK) return st;
  if (agg != nullptr) {
    fopd_aggregate<<<1, kSegThreads, 0, s>>>(f64, nws, nrws, lag, cu, B, agg);
    if ((st = launched()) != FOPD_OK) return st;
  }
  return FOPD_OK;
}

fopd_status fopd_loss_fwd_bwd(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                              const int32_t* token_ids, const uint8_t* mask, const float* behav_logp,
                              const float* teacher_logp, const float* teacher_logp_stale,
                              const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp,
                              const float* freshness_in, const int32_t* n_train_in, const int32_t* n_roll_in,
                              int64_t row_begin, const float* lse_in, const float* logp_in, float grad_scale,
                              float* loss,
                              float* freshness, float* weights, float* logp, void* dlogits,
                              void* workspace, size_t workspace_bytes, void* stream) {
  fopd_status st = loss_fwd_bwd_check_args(logits, dt, T, V, ld, token_ids, behav_logp, teacher_logp, seq_lens, lag, B,
                                           hp, freshness_in, n_train_in, n_roll_in, row_begin, lse_in, logp_in, loss,
                                           dlogits);
  if (st != FOPD_OK) return st;
  if ((st = check_workspace(workspace, workspace_bytes, T, B)) != FOPD_OK) return st;
  return loss_fwd_bwd_checked(logits, dt, T, V, ld, token_ids, mask, behav_logp, teacher_logp, teacher_logp_stale,
                              seq_lens, lag, B, hp, freshness_in, n_train_in, n_roll_in, row_begin, lse_in, logp_in,
                              grad_scale, loss, freshness, weights, logp, dlogits, workspace,
                              static_cast<hipStream_t>(stream), true);
}

fopd_status fopd_loss_fwd_bwd_unit(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                   const int32_t* token_ids, const uint8_t* mask, const float* behav_logp,
                                   const float* teacher_logp, const float* teacher_logp_stale,
                                   const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp,
                                   float grad_scale, float* loss, float* freshness, float* weights, float* logp,
                                   void* unit_rows, void* workspace, size_t workspace_bytes, void* stream) {
  fopd_status st = loss_fwd_bwd_check_args(logits, dt, T, V, ld, token_ids, behav_logp, teacher_logp, seq_lens, lag, B,
                                           hp, nullptr, nullptr, nullptr, 0, nullptr, nullptr, loss, unit_rows);
  if (st != FOPD_OK) return st;
  if ((st = check_workspace(workspace, workspace_bytes, T, B)) != FOPD_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Workspace w(T, B);
  int32_t* flags = at<int32_t>(workspace, w.flags);
  int64_t* cu = at<int64_t>(workspace, w.cu);
  int32_t* nws = at<int32_t>(workspace, w.n_train);
  int32_t* nrws = at<int32_t>(workspace, w.n_roll);
  double* f64 = at<double>(workspace, w.fresh64);
  float* coef = at<float>(workspace, w.coef);
  float* logp_ws = (logp != nullptr) ? logp : at<float>(workspace, w.logp);
  double* partials = at<double>(workspace, w.partials);

  fopd_scan_seqlens<<<1, kScanThreads, 0, s>>>(seq_lens, lag, B, T, T, cu, flags);
  if ((st = launched()) != FOPD_OK) return st;
  fopd_count_train<<<B, kSegThreads, 0, s>>>(mask, cu, T, nws, nrws);
  if ((st = launched()) != FOPD_OK) return st;
  // the one pass over the logits: log-probs and the rows at unit weight (no scores: fresh32 == nullptr)
  const RowPassArgs a{token_ids, mask, behav_logp, teacher_logp, cu, nws, nrws, lag, nullptr, B,
                      0, hp, grad_scale, logp_ws, partials, flags};
  if ((st = launch_k14(logits, unit_rows, dt, T, V, ld, a, s, true)) != FOPD_OK) return st;
  // scores, weights and the loss from the log-probs, exactly as the two-pass call forms them
  fopd_segment_stats<<<B, kSegThreads, 0, s>>>(logp_ws, behav_logp, nullptr, nullptr, teacher_logp, teacher_logp_stale,
                                               mask, cu, lag, T, hp, nullptr, nullptr, nullptr, nullptr, nullptr,
                                               nullptr, nullptr, nullptr, f64, nws, nrws);
  if ((st = launched()) != FOPD_OK) return st;
  const int64_t nblk = (T + kStreamThreads - 1) / kStreamThreads;
  if (T > 0) {
    fopd_coef_loss<<<static_cast<unsigned>(nblk), kStreamThreads, 0, s>>>(
        logp_ws, behav_logp, teacher_logp, mask, cu, nws, nrws, lag, f64, nullptr, T, B, 0, hp, grad_scale, coef,
        partials, flags);
    if ((st = launched()) != FOPD_OK) return st;
  }
  fopd_loss_final<<<1, kSegThreads, 0, s>>>(partials, nblk, nws, nrws, lag, f64, nullptr, B, hp.xi, loss, weights,
                                            freshness);
  return launched();
}

fopd_status fopd_loss_fwd_bwd_static(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                     const int32_t* token_ids, const uint8_t* mask, const float* behav_logp,
                                     const float* teacher_logp, const float* teacher_logp_stale,
                                     const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp,
                                     const float* freshness_in, const int32_t* n_train_in, const int32_t* n_roll_in,
                                     int64_t row_begin, const float* lse_in, const float* logp_in, float grad_scale,
                                     float* loss, float* freshness, float* weights, float* logp, void* dlogits,
                                     int32_t* flags_out, void* stream) {
  fopd_status st = loss_fwd_bwd_check_args(logits, dt, T, V, ld, token_ids, behav_logp, teacher_logp, seq_lens, lag, B,
                                           hp, freshness_in, n_train_in, n_roll_in, row_begin, lse_in, logp_in, loss,
                                           dlogits);
  if (st != FOPD_OK) return st;
  if (T > kStaticMaxRows || B > kStaticMaxSamples) return FOPD_ELIMIT;
  void* ws = nullptr;
  if ((st = static_scratch(&ws)) != FOPD_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // the array keeps the previous call's contents; only the flag words must start at zero (every other
  // region is written before it is read), and they are cleared by a kernel, not a memset
  fopd_clear_flags<<<1, 64, 0, s>>>(static_cast<int32_t*>(ws));
  if ((st = launched()) != FOPD_OK) return st;
  st = loss_fwd_bwd_checked(logits, dt, T, V, ld, token_ids, mask, behav_logp, teacher_logp, teacher_logp_stale,
                            seq_lens, lag, B, hp, freshness_in, n_train_in, n_roll_in, row_begin, lse_in, logp_in,
                            grad_scale, loss, freshness, weights, logp, dlogits, ws, s, false);
  if (st != FOPD_OK) return st;
  if (flags_out != nullptr) {
    fopd_copy_flags<<<1, 64, 0, s>>>(static_cast<const int32_t*>(ws), flags_out);
    st = launched();
  }
  return st;
}

fopd_status fopd_rollout_kl(const void* logits, const void* logits_stale, fopd_dtype dt, int64_t T, int64_t V,
                            int64_t ld, int64_t ld_stale, const int32_t* token_ids, const uint8_t* mask,
                            float* roll_kl, float* logp, float* lse, float* dlse, float* logq, void* workspace,
                            size_t workspace_bytes, void* stream) {
  fopd_status st = check_matrix(logits, dt, T, V, ld);
  if (st != FOPD_OK) return st;
  if ((st = check_matrix(logits_stale, dt, T, V, ld_stale)) != FOPD_OK) return st;
  if (token_ids == nullptr || roll_kl == nullptr || logp == nullptr || lse == nullptr || dlse == nullptr)
    return FOPD_EINVAL;
  if ((st = check_workspace(workspace, workspace_bytes, T, 0)) != FOPD_OK) return st;
  if (T == 0) return FOPD_OK;
  Workspace w(T, 0);
  hipStream_t s = static_cast<hipStream_t>(stream);
  ScopedTimer timer(0, s);
  const dim3 grid(static_cast<unsigned>(T)), block(kStreamThreads);
  if (dt == FOPD_BF16)
    fopd_k5_kl<FOPD_BF16, kUnroll><<<grid, block, 0, s>>>(logits, logits_stale, T, static_cast<int>(V), ld, ld_stale,
                                                          token_ids, mask, roll_kl, logp, lse, dlse, logq,
                                                          at<int32_t>(workspace, w.flags));
  else
    fopd_k5_kl<FOPD_F32, kUnroll><<<grid, block, 0, s>>>(logits, logits_stale, T, static_cast<int>(V), ld, ld_stale,
                                                         token_ids, mask, roll_kl, logp, lse, dlse, logq,
                                                         at<int32_t>(workspace, w.flags));
  return launched();
}

// The two-tensor variants share everything but the meaning of the second tensor.
//   teacher = false  second = stale checkpoint's logits: token_kl is the rollout drift; lq comes from the caller
//   teacher = true   second = teacher's logits: token_kl is the token loss; lq is read off the second tensor
// Whole-sample call (freshness_in == NULL): offsets, the pass over both tensors, scores, coefficients, loss,
// gradient.  Chunk call: the per-row results of fopd_rollout_kl and the scores of fopd_freshness_score come in,
// and only coefficients, the chunk's share of the loss and the gradient rows are made.
static fopd_status two_tensor_call(bool teacher, const void* logits, const void* second, fopd_dtype dt, int64_t T,
                                   int64_t V, int64_t ld, int64_t ld_second, const int32_t* token_ids,
                                   const uint8_t* mask, const float* behav_logp, const float* teacher_logp,
                                   const float* teacher_logp_stale, const int32_t* seq_lens, const int32_t* lag,
                                   int32_t B, fopd_hparams hp, const float* freshness_in, const int32_t* n_train_in,
                                   const int32_t* n_roll_in, int64_t row_begin, const float* lse_in,
                                   const float* logp_in, const float* dlse_in, const float* token_kl_in,
                                   float grad_scale, float* loss, float* freshness, float* weights, float* logp,
                                   float* token_kl, void* dlogits, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  fopd_status st = check_matrix(logits, dt, T, V, ld);
  if (st != FOPD_OK) return st;
  if ((st = check_matrix(second, dt, T, V, ld_second)) != FOPD_OK) return st;
  if ((st = check_matrix(dlogits, dt, T, V, ld)) != FOPD_OK) return st;
  if (B <= 0 || row_begin < 0) return FOPD_ESHAPE;
  if (token_ids == nullptr || seq_lens == nullptr || lag == nullptr || loss == nullptr) return FOPD_EINVAL;
  if (teacher ? (behav_logp == nullptr) : (teacher_logp == nullptr)) return FOPD_EINVAL;
  if (!(hp.alpha >= 0.f) || !(hp.beta >= 0.f)) return FOPD_EINVAL;
  if (dlogits == second) return FOPD_EINVAL;            // the second tensor is read by both passes
  const bool chunk = (freshness_in != nullptr);
  const bool all_in = n_train_in != nullptr && lse_in != nullptr && logp_in != nullptr && dlse_in != nullptr &&
                      token_kl_in != nullptr;
  const bool none_in = n_train_in == nullptr && n_roll_in == nullptr && lse_in == nullptr && logp_in == nullptr &&
                       dlse_in == nullptr && token_kl_in == nullptr && row_begin == 0;
  if (chunk ? !all_in : !none_in) return FOPD_EINVAL;
  if ((st = check_workspace(workspace, workspace_bytes, T, B)) != FOPD_OK) return st;

  const Workspace w(T, B);
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* flags = at<int32_t>(workspace, w.flags);
  int64_t* cu = at<int64_t>(workspace, w.cu);
  int32_t* nws = at<int32_t>(workspace, w.n_train);
  int32_t* nrws = at<int32_t>(workspace, w.n_roll);
  double* f64 = at<double>(workspace, w.fresh64);
  float* c1 = at<float>(workspace, w.coef);
  float* c2 = at<float>(workspace, w.coef2);
  double* partials = at<double>(workspace, w.partials);

  fopd_scan_seqlens<<<1, kScanThreads, 0, s>>>(seq_lens, lag, B, chunk ? -1 : T, row_begin + T, cu, flags);
  if ((st = launched()) != FOPD_OK) return st;

  const float* lse_use = lse_in;
  const float* logp_use = logp_in;
  const float* dlse_use = dlse_in;
  const float* kl_use = token_kl_in;
  const int32_t* n_use = n_train_in;
  const int32_t* nr_use = (n_roll_in != nullptr) ? n_roll_in : n_train_in;
  const double* f64_use = nullptr;
  const float* lq_use = teacher_logp;
  if (!chunk) {
    float* lse_ws = at<float>(workspace, w.lse);
    float* dlse_ws = at<float>(workspace, w.dlse);
    float* logq_ws = at<float>(workspace, w.logq);
    float* logp_ws = (logp != nullptr) ? logp : at<float>(workspace, w.logp);
    float* kl_ws = (token_kl != nullptr) ? token_kl : at<float>(workspace, w.kl);
    st = fopd_rollout_kl(logits, second, dt, T, V, ld, ld_second, token_ids, mask, kl_ws, logp_ws, lse_ws, dlse_ws,
                         teacher ? logq_ws : nullptr, workspace, workspace_bytes, stream);
    if (st != FOPD_OK) return st;
    if (teacher) lq_use = logq_ws;      // the teacher's log-prob of the sampled token, for D^sup
    // stale tensor: drift = the full KL, token loss = sampled form; teacher tensor: the other way round
    fopd_segment_stats<<<B, kSegThreads, 0, s>>>(logp_ws, behav_logp, teacher ? nullptr : kl_ws,
                                                 teacher ? kl_ws : nullptr, lq_use, teacher_logp_stale, mask, cu, lag,
                                                 T, hp, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                                 nullptr, f64, nws, nrws);
    if ((st = launched()) != FOPD_OK) return st;
    lse_use = lse_ws;
    logp_use = logp_ws;
    dlse_use = dlse_ws;
    kl_use = kl_ws;
    n_use = nws;
    nr_use = nrws;
    f64_use = f64;
  } else {
    if (logp != nullptr && logp != logp_in && T > 0 &&
        hipMemcpyAsync(logp, logp_in, static_cast<size_t>(T) * sizeof(float), hipMemcpyDeviceToDevice, s) != hipSuccess)
      return FOPD_EHIP;
    if (token_kl != nullptr && token_kl != token_kl_in && T > 0 &&
        hipMemcpyAsync(token_kl, token_kl_in, static_cast<size_t>(T) * sizeof(float), hipMemcpyDeviceToDevice, s) !=
            hipSuccess)
      return FOPD_EHIP;
  }

  const int64_t nblk = (T + kStreamThreads - 1) / kStreamThreads;
  if (T > 0) {
    fopd_coef_loss_kl<<<static_cast<unsigned>(nblk), kStreamThreads, 0, s>>>(
        logp_use, kl_use, lq_use, behav_logp, mask, cu, n_use, nr_use, lag, f64_use, freshness_in, T, B, row_begin, hp,
        grad_scale, !teacher, c1, c2, partials);
    if ((st = launched()) != FOPD_OK) return st;
  }
  fopd_loss_final<<<1, kSegThreads, 0, s>>>(partials, nblk, n_use, nr_use, lag, f64_use, freshness_in, B, hp.xi, loss,
                                            weights, freshness);
  if ((st = launched()) != FOPD_OK) return st;
  if (T == 0) return FOPD_OK;
  ScopedTimer timer(1, s);
  const dim3 grid(static_cast<unsigned>(T)), block(kStreamThreads);
  if (dt == FOPD_BF16)
    fopd_k6_grad_kl<FOPD_BF16, kUnroll><<<grid, block, 0, s>>>(logits, second, dlogits, T, static_cast<int>(V), ld,
                                                               ld_second, token_ids, lse_use, dlse_use, kl_use, logp_use,
                                                               c1, c2);
  else
    fopd_k6_grad_kl<FOPD_F32, kUnroll><<<grid, block, 0, s>>>(logits, second, dlogits, T, static_cast<int>(V), ld,
                                                              ld_second, token_ids, lse_use, dlse_use, kl_use, logp_use,
                                                              c1, c2);
  return launched();
}

fopd_status fopd_loss_fwd_bwd_full_kl(const void* logits, const void* logits_stale, fopd_dtype dt, int64_t T,
                                      int64_t V, int64_t ld, int64_t ld_stale, const int32_t* token_ids,
                                      const uint8_t* mask, const float* teacher_logp,
                                      const float* teacher_logp_stale, const int32_t* seq_lens, const int32_t* lag,
                                      int32_t B, fopd_hparams hp, const float* freshness_in,
                                      const int32_t* n_train_in, const int32_t* n_roll_in, int64_t row_begin,
                                      const float* lse_in, const float* logp_in, const float* dlse_in,
                                      const float* roll_kl_in, float grad_scale, float* loss, float* freshness,
                                      float* weights, float* logp, float* roll_kl, void* dlogits, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  return two_tensor_call(false, logits, logits_stale, dt, T, V, ld, ld_stale, token_ids, mask, nullptr, teacher_logp,
                         teacher_logp_stale, seq_lens, lag, B, hp, freshness_in, n_train_in, n_roll_in, row_begin,
                         lse_in, logp_in, dlse_in, roll_kl_in, grad_scale, loss, freshness, weights, logp, roll_kl,
                         dlogits, workspace, workspace_bytes, stream);
}

fopd_status fopd_loss_fwd_bwd_full_teacher(const void* logits, const void* teacher_logits, fopd_dtype dt, int64_t T,
                                           int64_t V, int64_t ld, int64_t ld_teacher, const int32_t* token_ids,
                                           const uint8_t* mask, const float* behav_logp,
                                           const float* teacher_logp_stale, const int32_t* seq_lens,
                                           const int32_t* lag, int32_t B, fopd_hparams hp, const float* freshness_in,
                                           const int32_t* n_train_in, const int32_t* n_roll_in, int64_t row_begin,
                                           const float* lse_in, const float* logp_in, const float* dlse_in,
                                           const float* token_kl_in, float grad_scale, float* loss, float* freshness,
                                           float* weights, float* logp, float* token_kl, void* dlogits,
                                           void* workspace, size_t workspace_bytes, void* stream) {
  return two_tensor_call(true, logits, teacher_logits, dt, T, V, ld, ld_teacher, token_ids, mask, behav_logp, nullptr,
                         teacher_logp_stale, seq_lens, lag, B, hp, freshness_in, n_train_in, n_roll_in, row_begin,
                         lse_in, logp_in, dlse_in, token_kl_in, grad_scale, loss, freshness, weights, logp, token_kl,
                         dlogits, workspace, workspace_bytes, stream);
}

size_t fopd_topk_workspace_bytes(int64_t T, int32_t B, int32_t k) {
  const size_t t = static_cast<size_t>(T < 0 ? 0 : T), kk = static_cast<size_t>(k < 0 ? 0 : k);
  return Workspace(T, B).total + 2 * align_up(t * kk * sizeof(float), 256);
}

static fopd_status launch_topk_terms(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                     const int32_t* token_ids, const uint8_t* mask, const int32_t* list_ids,
                                     const float* list_logp, int32_t k, float rest_floor, const float* lse,
                                     float* token_loss, float* g_rest, float* p_list, float* h_list, hipStream_t s) {
  if (T == 0) return FOPD_OK;
  const dim3 grid(static_cast<unsigned>((T + kListRows - 1) / kListRows)), block(kListThreads);
  if (dt == FOPD_BF16)
    fopd_topk_terms<FOPD_BF16><<<grid, block, 0, s>>>(logits, T, static_cast<int>(V), ld, token_ids, mask, list_ids,
                                                     list_logp, k, rest_floor, lse, token_loss, g_rest, p_list, h_list);
  else
    fopd_topk_terms<FOPD_F32><<<grid, block, 0, s>>>(logits, T, static_cast<int>(V), ld, token_ids, mask, list_ids,
                                                    list_logp, k, rest_floor, lse, token_loss, g_rest, p_list, h_list);
  return launched();
}

fopd_status fopd_topk_token_loss(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                 const int32_t* token_ids, const uint8_t* mask, const int32_t* list_ids,
                                 const float* list_logp, int32_t k, float rest_floor, const float* lse,
                                 float* token_loss, void* stream) {
  fopd_status st = check_matrix(logits, dt, T, V, ld);
  if (st != FOPD_OK) return st;
  if (k < 1 || k > 4096) return FOPD_ESHAPE;
  if (token_ids == nullptr || list_ids == nullptr || list_logp == nullptr || lse == nullptr || token_loss == nullptr)
    return FOPD_EINVAL;
  if (!(rest_floor > 0.f) || !(rest_floor <= 1.f)) return FOPD_EINVAL;
  return launch_topk_terms(logits, dt, T, V, ld, token_ids, mask, list_ids, list_logp, k, rest_floor, lse, token_loss,
                           nullptr, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

fopd_status fopd_loss_fwd_bwd_topk_teacher(const void* logits, fopd_dtype dt, int64_t T, int64_t V, int64_t ld,
                                           const int32_t* token_ids, const uint8_t* mask, const float* behav_logp,
                                           const int32_t* list_ids, const float* list_logp, int32_t k,
                                           float rest_floor, const float* teacher_logp,
                                           const float* teacher_logp_stale, const int32_t* seq_lens,
                                           const int32_t* lag, int32_t B, fopd_hparams hp, const float* freshness_in,
                                           const int32_t* n_train_in, const int32_t* n_roll_in, int64_t row_begin,
                                           const float* lse_in, const float* logp_in, float grad_scale, float* loss,
                                           float* freshness, float* weights, float* logp, float* token_loss,
                                           void* dlogits, void* workspace, size_t workspace_bytes, void* stream) {
  fopd_status st = check_matrix(logits, dt, T, V, ld);
  if (st != FOPD_OK) return st;
  if ((st = check_matrix(dlogits, dt, T, V, ld)) != FOPD_OK) return st;
  if (B <= 0 || k < 1 || k > 4096 || row_begin < 0) return FOPD_ESHAPE;
  if (token_ids == nullptr || behav_logp == nullptr || list_ids == nullptr || list_logp == nullptr ||
      seq_lens == nullptr || lag == nullptr || loss == nullptr)
    return FOPD_EINVAL;
  if (teacher_logp_stale != nullptr && teacher_logp == nullptr) return FOPD_EINVAL;
  if (!(rest_floor > 0.f) || !(rest_floor <= 1.f)) return FOPD_EINVAL;
  if (!(hp.alpha >= 0.f) || !(hp.beta >= 0.f)) return FOPD_EINVAL;
  // a chunk of a longer batch brings the scores, the counts and its slices of lse and logp; a whole batch none
  const bool chunk = (freshness_in != nullptr);
  const bool all_in = n_train_in != nullptr && lse_in != nullptr && logp_in != nullptr;
  const bool none_in = n_train_in == nullptr && n_roll_in == nullptr && lse_in == nullptr && logp_in == nullptr &&
                       row_begin == 0;
  if (chunk ? !all_in : !none_in) return FOPD_EINVAL;
  if ((st = check_workspace(workspace, workspace_bytes, T, B)) != FOPD_OK) return st;
  if (workspace_bytes < fopd_topk_workspace_bytes(T, B, k)) return FOPD_EWORKSPACE;

  const Workspace w(T, B);
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* flags = at<int32_t>(workspace, w.flags);
  int64_t* cu = at<int64_t>(workspace, w.cu);
  int32_t* nws = at<int32_t>(workspace, w.n_train);
  int32_t* nrws = at<int32_t>(workspace, w.n_roll);
  double* f64 = at<double>(workspace, w.fresh64);
  float* c1 = at<float>(workspace, w.coef);
  float* c2 = at<float>(workspace, w.coef2);
  float* tl_ws = (token_loss != nullptr) ? token_loss : at<float>(workspace, w.kl);
  float* g_rest = at<float>(workspace, w.dlse);
  float* row_coef = at<float>(workspace, w.logq);
  double* partials = at<double>(workspace, w.partials);
  const size_t list_bytes = align_up(static_cast<size_t>(T) * static_cast<size_t>(k) * sizeof(float), 256);
  float* p_list = at<float>(workspace, w.total);
  float* h_list = at<float>(workspace, w.total + list_bytes);

  fopd_scan_seqlens<<<1, kScanThreads, 0, s>>>(seq_lens, lag, B, chunk ? -1 : T, row_begin + T, cu, flags);
  if ((st = launched()) != FOPD_OK) return st;
  const float* lse_use = lse_in;
  const float* logp_use = logp_in;
  const int32_t* n_use = n_train_in;
  const int32_t* nr_use = (n_roll_in != nullptr) ? n_roll_in : n_train_in;
  const double* f64_use = nullptr;
  if (!chunk) {
    float* lse_ws = at<float>(workspace, w.lse);
    float* logp_ws = (logp != nullptr) ? logp : at<float>(workspace, w.logp);
    if ((st = launch_k1(logits, dt, T, V, ld, token_ids, mask, logp_ws, lse_ws, nullptr, nullptr, flags, s)) != FOPD_OK)
      return st;
    lse_use = lse_ws;
    logp_use = logp_ws;
  } else if (logp != nullptr && logp != logp_in && T > 0 &&
             hipMemcpyAsync(logp, logp_in, static_cast<size_t>(T) * sizeof(float), hipMemcpyDeviceToDevice, s) !=
                 hipSuccess) {
    return FOPD_EHIP;
  }
  if ((st = launch_topk_terms(logits, dt, T, V, ld, token_ids, mask, list_ids, list_logp, k, rest_floor, lse_use, tl_ws,
                              g_rest, p_list, h_list, s)) != FOPD_OK)
    return st;
  if (!chunk) {
    // token loss = the distribution-level value per row; rollout drift = the sampled estimator; D^sup from the two
    // sampled-token arrays when both are there
    fopd_segment_stats<<<B, kSegThreads, 0, s>>>(logp_use, behav_logp, nullptr, tl_ws, teacher_logp,
                                                 teacher_logp_stale, mask, cu, lag, T, hp, nullptr, nullptr, nullptr,
                                                 nullptr, nullptr, nullptr, nullptr, nullptr, f64, nws, nrws);
    if ((st = launched()) != FOPD_OK) return st;
    n_use = nws;
    nr_use = nrws;
    f64_use = f64;
  }
  const int64_t nblk = (T + kStreamThreads - 1) / kStreamThreads;
  if (T > 0) {
    fopd_coef_loss_kl<<<static_cast<unsigned>(nblk), kStreamThreads, 0, s>>>(
        logp_use, tl_ws, nullptr, behav_logp, mask, cu, n_use, nr_use, lag, f64_use, freshness_in, T, B, row_begin, hp,
        grad_scale, false, c1, c2, partials);
    if ((st = launched()) != FOPD_OK) return st;
  }
  fopd_loss_final<<<1, kSegThreads, 0, s>>>(partials, nblk, n_use, nr_use, lag, f64_use, freshness_in, B, hp.xi, loss,
                                            weights, freshness);
  if ((st = launched()) != FOPD_OK) return st;
  if (T == 0) return FOPD_OK;
  fopd_topk_row_coef<<<static_cast<unsigned>(nblk), kStreamThreads, 0, s>>>(c1, c2, g_rest, T, row_coef);
  if ((st = launched()) != FOPD_OK) return st;
  if ((st = launch_k4(logits, dlogits, dt, T, V, ld, token_ids, lse_use, logp_use, row_coef, s)) != FOPD_OK) return st;
  const dim3 grid(static_cast<unsigned>((T + kListRows - 1) / kListRows)), block(kListThreads);
  if (dt == FOPD_BF16)
    fopd_topk_fixup<FOPD_BF16><<<grid, block, 0, s>>>(dlogits, T, static_cast<int>(V), ld, token_ids, list_ids, k,
                                                     logp_use, c1, c2, g_rest, p_list, h_list, nullptr);
  else
    fopd_topk_fixup<FOPD_F32><<<grid, block, 0, s>>>(dlogits, T, static_cast<int>(V), ld, token_ids, list_ids, k,
                                                    logp_use, c1, c2, g_rest, p_list, h_list, nullptr);
  return launched();
}

int fopd_refresh_decide(const float* agg_host, const fopd_refresh_config* cfg_host, fopd_refresh_state* state_host,
                        int64_t step, int32_t* reason_host) {
  if (agg_host == nullptr || cfg_host == nullptr || state_host == nullptr || cfg_host->min_interval < 1) return -1;
  int32_t reason = 0;
  if (agg_host[0] <= cfg_host->kappa_f) reason |= 1;
  if (agg_host[1] < cfg_host->kappa_roll) reason |= 2;
  if (agg_host[2] < cfg_host->kappa_sup) reason |= 4;
  if (reason_host != nullptr) *reason_host = reason;
  if (reason == 0) return 0;
  const bool rested = state_host->last_refresh_step < 0 ||
                      step - state_host->last_refresh_step >= cfg_host->min_interval;
  if (!rested) return 0;
  state_host->last_refresh_step = step;
  state_host->refreshes += 1;
  return 1;
}

size_t fopd_lm_head_workspace_bytes(int64_t T) {
  return LmWorkspace(T).total;
}

fopd_status fopd_lm_head_token_logprobs(const void* hidden, int64_t ldh, const void* weight, int64_t ldw,
                                        int64_t T, int64_t V, int64_t d, const int32_t* token_ids,
                                        const uint8_t* mask, float* logp, float* lse, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  if (T < 0 || V <= 0 || d <= 0 || d % (2 * kLmK) != 0 || ldh < d || ldw < d) return FOPD_ESHAPE;
  // every byte offset inside the projection matrix must fit 32 bits
  if (V * ldw >= 2147483648LL || ldh >= 2147483648LL) return FOPD_ESHAPE;
  if (hidden == nullptr || weight == nullptr || token_ids == nullptr || logp == nullptr || lse == nullptr)
    return FOPD_EINVAL;
  // ... and inside the hidden states of one launch: more rows than that go through in blocks (rows are independent)
  if (T * ldh >= 2147483648LL) {
    if (misaligned(hidden, 16) || (ldh * 2) % 16 != 0) return FOPD_EALIGN;
    if (workspace == nullptr || misaligned(workspace, 256) || workspace_bytes < LmWorkspace(T).total)
      return FOPD_EWORKSPACE;
    const int64_t block = (2147483647LL / ldh) / kLmTile * kLmTile;
    if (block <= 0) return FOPD_ESHAPE;
    for (int64_t a = 0; a < T; a += block) {
      const int64_t rows = (T - a < block) ? T - a : block;
      const fopd_status st = fopd_lm_head_token_logprobs(
          static_cast<const __bf16*>(hidden) + a * ldh, ldh, weight, ldw, rows, V, d, token_ids + a,
          mask == nullptr ? nullptr : mask + a, logp + a, lse + a, workspace, workspace_bytes, stream);
      if (st != FOPD_OK) return st;
    }
    return FOPD_OK;
  }
  if (misaligned(hidden, 16) || misaligned(weight, 16) || (ldh * 2) % 16 != 0 || (ldw * 2) % 16 != 0)
    return FOPD_EALIGN;
  const LmWorkspace lay(T);
  if (workspace == nullptr || misaligned(workspace, 256) || workspace_bytes < lay.total) return FOPD_EWORKSPACE;
  if (T == 0) return FOPD_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  auto kern = fopd_k7_lm_head_lse;
  static bool allowed[kMaxDevices] = {};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), kLmLdsBytes, allowed) != FOPD_OK) return FOPD_EHIP;
  const int n_token_tiles = static_cast<int>(lay.t_pad / kLmTile);
  const int n_vocab_tiles = static_cast<int>((V + kLmTile - 1) / kLmTile);
  // strips: 8, 16 or 32, whichever leaves the smallest idle tail when the work items (token tile x strip,
  // all of one length) are dealt to the 256 compute units round by round
  int n_strips = 8;
  double best = 0.0;
  for (int cand = 8; cand <= kLmStripsMax; cand *= 2) {
    const int64_t items = static_cast<int64_t>(n_token_tiles) * cand;
    const double fill = static_cast<double>(items) / static_cast<double>((items + 255) / 256 * 256);
    if (fill > best + 0.005) {
      best = fill;
      n_strips = cand;
    }
  }
  const unsigned grid = static_cast<unsigned>((n_token_tiles + 31) / 32) * static_cast<unsigned>(n_strips / 8) * 256u;
  float2* partial = at<float2>(workspace, lay.partial);
  const __bf16* Wp = static_cast<const __bf16*>(weight);
  const __bf16* Hp = static_cast<const __bf16*>(hidden);
  // Masked rows have no log-prob: with a mask only the other rows are projected.  Their count stays on the device;
  // the kernel gathers them through a row map as it loads and leaves out the token tiles past the count.
  int32_t *ex = nullptr, *row_map = nullptr, *n_live = nullptr;
  if (mask != nullptr && current_options().lm_head_compact != 0) {
    ex = at<int32_t>(workspace, lay.ex);
    row_map = at<int32_t>(workspace, lay.row_map);
    n_live = at<int32_t>(workspace, lay.n_live);
    fopd_live_scan<<<1, kLiveScanThreads, 0, s>>>(mask, nullptr, nullptr, static_cast<int>(T), nullptr, -1, 0, ex, row_map,
                                                  n_live, nullptr, nullptr);
    if (launched() != FOPD_OK) return FOPD_EHIP;
  }
  {
    ScopedTimer timer(3, s);
    kern<<<dim3(grid), dim3(kLmThreads), kLmLdsBytes, s>>>(Wp, ldw, Hp, ldh, static_cast<int>(T), static_cast<int>(V),
                                                    static_cast<int>(d), partial, n_token_tiles, n_vocab_tiles,
                                                    n_strips, static_cast<int64_t>(lay.t_pad), row_map, n_live);
  }
  if (launched() != FOPD_OK) return FOPD_EHIP;
  fopd_k7_finish<<<dim3(static_cast<unsigned>((T + 3) / 4)), dim3(256), 0, s>>>(
      Wp, ldw, Hp, ldh, partial, n_strips, static_cast<int>(T), static_cast<int>(V), static_cast<int>(d),
      static_cast<int64_t>(lay.t_pad), token_ids, mask, logp, lse, at<int32_t>(workspace, lay.flags), ex);
  return launched();
}

size_t fopd_lm_head_loss_workspace_bytes(int64_t T, int64_t V, int64_t d, int32_t B, int64_t rows_chunk) {
  return LmLossWorkspace(T, V, d, B, rows_chunk).total;
}

// Out[n, m] (+)= sum_k Bn[n, k] Am[m, k] on `s`; `slot` = timing slot of this contraction.  n_live != NULL: a device
// int, the number of leading rows of Bn that count (the tiles past them are not computed).
static fopd_status launch_gemm(bool accumulate, const __bf16* Am, int64_t lda, int64_t M, const __bf16* Bn, int64_t ldb,
                               int64_t N, int64_t K, float* Out, int64_t ldo, int slot, hipStream_t s,
                               const int* n_live = nullptr) {
  if (M <= 0 || N <= 0) return FOPD_OK;
  if (K <= 0 || K % 64 != 0 || M > 2147483647LL || N > 2147483647LL || K > 2147483647LL) return FOPD_ESHAPE;
  // byte offsets inside one 256-row operand tile are 32-bit
  if (256 * lda * 2 >= 2147483648LL || 256 * ldb * 2 >= 2147483648LL) return FOPD_ESHAPE;
  static bool allowed[2][kMaxDevices] = {};
  const void* kern = accumulate ? reinterpret_cast<const void*>(fopd_gemm_nt<true, 0>)
                                : reinterpret_cast<const void*>(fopd_gemm_nt<false, 0>);
  if (allow_dynamic_lds(kern, kGemmLdsBytes, allowed[accumulate ? 1 : 0]) != FOPD_OK) return FOPD_EHIP;
  const int tiles_m = static_cast<int>((M + kGemmTile - 1) / kGemmTile);
  const int tiles_n = static_cast<int>((N + kGemmTileN - 1) / kGemmTileN);
  const int64_t rounds = static_cast<int64_t>((tiles_m + 7) / 8) * ((tiles_n + 31) / 32);
  if (rounds * 256 > 2147483647LL) return FOPD_ESHAPE;
  const dim3 grid(static_cast<unsigned>(rounds * 256)), block(kGemmThreads);
  ScopedTimer timer(slot, s);
  if (accumulate)
    fopd_gemm_nt<true, 0><<<grid, block, kGemmLdsBytes, s>>>(Am, lda, static_cast<int>(M), Bn, ldb, static_cast<int>(N),
                                                          static_cast<int>(K), Out, ldo, tiles_m, tiles_n, n_live);
  else
    fopd_gemm_nt<false, 0><<<grid, block, kGemmLdsBytes, s>>>(Am, lda, static_cast<int>(M), Bn, ldb, static_cast<int>(N),
                                                           static_cast<int>(K), Out, ldo, tiles_m, tiles_n, n_live);
  return launched();
}

// Out[n, m] (+)= sum_{k < K} Bk[k, n] Ak[k, m] on `s`; Ak has rows_a readable rows, Bk has K and zeros where a row
// is not to count.  k_live != NULL: a device int, the number of leading rows that count (K is cut to it, rounded up to 64).
static fopd_status launch_gemm_tn(bool accumulate, const __bf16* Ak, int64_t lda, int64_t M, int64_t rows_a,
                                  const __bf16* Bk, int64_t ldb, int64_t N, int64_t K, float* Out, int64_t ldo, int slot,
                                  hipStream_t s, const int* k_live = nullptr) {
  if (M <= 0 || N <= 0) return FOPD_OK;
  if (K <= 0 || K % 64 != 0 || rows_a < 1 || rows_a > K || M > 2147483647LL || N > 2147483647LL || K > 2147483647LL ||
      M % 8 != 0 || lda % 8 != 0 || ldb % 8 != 0 || lda < M || ldb < (N + 7) / 8 * 8)
    return FOPD_ESHAPE;
  static bool allowed[2][kMaxDevices] = {};
  const void* kern = accumulate ? reinterpret_cast<const void*>(fopd_gemm_tn<true>)
                                : reinterpret_cast<const void*>(fopd_gemm_tn<false>);
  if (allow_dynamic_lds(kern, kTnLdsBytes, allowed[accumulate ? 1 : 0]) != FOPD_OK) return FOPD_EHIP;
  const int tiles_m = static_cast<int>((M + kGemmTile - 1) / kGemmTile);
  const int tiles_n = static_cast<int>((N + kGemmTileN - 1) / kGemmTileN);
  const int64_t rounds = static_cast<int64_t>((tiles_m + 7) / 8) * ((tiles_n + 31) / 32);
  if (rounds * 256 > 2147483647LL) return FOPD_ESHAPE;
  const dim3 grid(static_cast<unsigned>(rounds * 256)), block(kGemmThreads);
  ScopedTimer timer(slot, s);
  if (accumulate)
    fopd_gemm_tn<true><<<grid, block, kTnLdsBytes, s>>>(Ak, lda, static_cast<int>(M), static_cast<int>(rows_a), Bk, ldb,
                                                       static_cast<int>(N), static_cast<int>(K), Out, ldo, tiles_m,
                                                       tiles_n, k_live);
  else
    fopd_gemm_tn<false><<<grid, block, kTnLdsBytes, s>>>(Ak, lda, static_cast<int>(M), static_cast<int>(rows_a), Bk, ldb,
                                                        static_cast<int>(N), static_cast<int>(K), Out, ldo, tiles_m,
                                                        tiles_n, k_live);
  return launched();
}

static fopd_status launch_transpose(const void* in, int64_t ld_in, int64_t rows, int64_t cols, void* out, int64_t ld_out,
                                    int64_t rows_pad, hipStream_t s) {
  if (rows_pad <= 0 || cols <= 0) return FOPD_OK;
  const dim3 grid(static_cast<unsigned>((rows_pad + 63) / 64), static_cast<unsigned>((cols + 63) / 64));
  if (grid.y > 65535u) {      // the second grid dimension is short: walk it in slabs
    for (int64_t c0 = 0; c0 < cols; c0 += 65535LL * 64) {
      const int64_t cn = (cols - c0 < 65535LL * 64) ? cols - c0 : 65535LL * 64;
      const dim3 g2(grid.x, static_cast<unsigned>((cn + 63) / 64));
      fopd_transpose_bf16<<<g2, 256, 0, s>>>(static_cast<const uint16_t*>(in) + c0, ld_in, static_cast<int>(rows),
                                             static_cast<int>(cn), static_cast<uint16_t*>(out) + c0 * ld_out, ld_out,
                                             static_cast<int>(rows_pad));
      if (launched() != FOPD_OK) return FOPD_EHIP;
    }
    return FOPD_OK;
  }
  fopd_transpose_bf16<<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(in), ld_in, static_cast<int>(rows),
                                           static_cast<int>(cols), static_cast<uint16_t*>(out), ld_out,
                                           static_cast<int>(rows_pad));
  return launched();
}

// The loss pass through the projection.  `listed` == nullptr: the sampled-token loss against teacher_logp
// (fopd_lm_head_loss_fwd_bwd); else the distribution-level loss against a teacher stored as k tokens per row, scores
// formed inside the call (fopd_lm_head_loss_fwd_bwd_topk_teacher; teacher_logp then only serves D^sup and may be NULL).
static fopd_status lm_head_loss_impl(const void* hidden, int64_t ldh, const void* weight, int64_t ldw, int64_t T,
                                     int64_t V, int64_t d, const int32_t* token_ids, const uint8_t* mask,
                                     const float* behav_logp, const float* teacher_logp, const int32_t* seq_lens,
                                     const int32_t* lag, int32_t B, fopd_hparams hp, const float* freshness_in,
                                     const int32_t* n_train_in, const int32_t* n_roll_in,
                                     const int32_t* seq_lens_host, float grad_scale, int64_t rows_chunk, float* loss,
                                     float* freshness, float* weights, float* logp, float* lse, float* dhidden,
                                     int64_t lddh, float* dweight, int64_t lddw, int accumulate_dweight,
                                     const ListedTeacher* listed, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  // without the two gradient outputs the call only scores: log-probs, token loss, scores, weights and the loss
  // (first loop of Algorithm 1 on projected logits)
  const bool grads = (dhidden != nullptr);
  const bool head_grad = (dweight != nullptr);         // NULL with dhidden given: the projection is not trained
  if (T < 0 || T > 2147483647LL || V <= 0 || V > 2147483647LL - 64 || d <= 0 || d % 64 != 0 || ldh < d || ldw < d ||
      (grads && lddh < d) || (head_grad && lddw < d) || B <= 0 || rows_chunk < 64 || rows_chunk % 64 != 0 || rows_chunk > 1048576)
    return FOPD_ESHAPE;
  if (hidden == nullptr || weight == nullptr || token_ids == nullptr || behav_logp == nullptr ||
      (teacher_logp == nullptr && listed == nullptr) || seq_lens == nullptr || lag == nullptr || loss == nullptr ||
      (logp == nullptr) != (lse == nullptr) || (dhidden == nullptr && dweight != nullptr))
    return FOPD_EINVAL;
  // Without the two per-row outputs (a caller that supplies scores has them from the scoring call) the samples of
  // weight 0 are left out of the call altogether; this needs the scores and the numbering of the live rows.
  const bool drop_gated = (logp == nullptr);
  if (drop_gated && (freshness_in == nullptr || listed != nullptr || dhidden == nullptr ||
                     current_options().lm_head_compact == 0))
    return FOPD_EINVAL;
  if (!grads && freshness_in != nullptr) return FOPD_EINVAL;       // scoring needs the scores to be formed inside
  if (listed != nullptr) {
    if (listed->k < 1 || listed->k > 4096) return FOPD_ESHAPE;
    if (listed->ids == nullptr || listed->logp == nullptr) return FOPD_EINVAL;
    if (listed->teacher_logp_stale != nullptr && teacher_logp == nullptr) return FOPD_EINVAL;
    if (!(listed->rest_floor > 0.f) || !(listed->rest_floor <= 1.f)) return FOPD_EINVAL;
  }
  const int32_t list_k = (listed != nullptr) ? listed->k : 0;
  const bool scored = (freshness_in != nullptr);
  // without scores they are formed inside the call, per chunk: the chunks then follow sample boundaries, which
  // the host must know
  if (!scored && (seq_lens_host == nullptr || n_train_in != nullptr || n_roll_in != nullptr)) return FOPD_EINVAL;
  if (n_roll_in != nullptr && n_train_in == nullptr) return FOPD_EINVAL;
  if (!(hp.alpha >= 0.f) || !(hp.beta >= 0.f)) return FOPD_EINVAL;
  if (misaligned(hidden, 16) || misaligned(weight, 16) || (ldh * 2) % 16 != 0 || (ldw * 2) % 16 != 0 ||
      misaligned(dhidden, 16) || misaligned(dweight, 16))
    return FOPD_EALIGN;
  const LmLossWorkspace lay(T, V, d, B, rows_chunk, list_k);
  if (workspace == nullptr || misaligned(workspace, 256) || workspace_bytes < lay.total) return FOPD_EWORKSPACE;

  // The chunks: [row begin, rows, first sample, one past the last sample].  With scores supplied they are
  // rows_chunk rows each and may cut samples; without, whole samples are gathered up to rows_chunk rows.  Without
  // scores and with a sample that does not fit into a chunk, the call sweeps the rows twice in chunks of rows_chunk
  // rows: first only logits and log-probs (one contraction per chunk), then, with the scores of all samples known,
  // the pass proper as if the scores had been supplied.
  struct Chunk {
    int64_t a, R;
    int32_t i0, i1;
  };
  std::vector<Chunk> chunks;
  bool two_sweeps = false;
  if (!scored) {
    int64_t total = 0;
    for (int32_t i = 0; i < B; ++i) {
      const int64_t len = seq_lens_host[i];
      if (len < 0) return FOPD_ESHAPE;
      if (len > rows_chunk) two_sweeps = true;
      total += len;
    }
    if (total != T) return FOPD_ESHAPE;                          // the lengths must add up to T
  }
  const bool fixed = scored || two_sweeps;                       // chunks of rows_chunk rows that may cut samples
  if (fixed) {
    for (int64_t a = 0; a < T; a += rows_chunk) chunks.push_back({a, (T - a < rows_chunk) ? T - a : rows_chunk, 0, 0});
  } else {
    int64_t a = 0, rows = 0;
    int32_t i0 = 0;
    for (int32_t i = 0; i < B; ++i) {
      const int64_t len = seq_lens_host[i];
      if (rows + len > rows_chunk) {
        chunks.push_back({a, rows, i0, i});
        a += rows;
        rows = 0;
        i0 = i;
      }
      rows += len;
    }
    if (a + rows != T) return FOPD_ESHAPE;                       // the lengths must add up to T
    if (rows > 0) chunks.push_back({a, rows, i0, B});
    else if (!chunks.empty()) chunks.back().i1 = B;              // trailing empty samples
  }

  hipStream_t s = static_cast<hipStream_t>(stream);
  fopd_status st;
  int32_t* flags = at<int32_t>(workspace, lay.flags);
  int64_t* cu = at<int64_t>(workspace, lay.cu);
  int32_t* nws = at<int32_t>(workspace, lay.n_train);
  int32_t* nrws = at<int32_t>(workspace, lay.n_roll);
  double* f64 = at<double>(workspace, lay.fresh64);
  float* coef = at<float>(workspace, lay.coef);
  double* partials = at<double>(workspace, lay.partials);
  float* chunk_loss = at<float>(workspace, lay.chunk_loss);
  float* Z = at<float>(workspace, lay.z);
  __bf16* G = at<__bf16>(workspace, lay.g);
  __bf16* Wt = at<__bf16>(workspace, lay.wt);
  const __bf16* Hm = static_cast<const __bf16*>(hidden);
  const __bf16* Wm = static_cast<const __bf16*>(weight);
  const int64_t ldz = lay.ldz;
  const double* f64_use = scored ? nullptr : f64;
  float* tl = nullptr;               // listed teacher: token loss of every row, then this chunk's per-row values
  float *c2 = nullptr, *g_rest = nullptr, *row_coef = nullptr, *p_list = nullptr, *h_list = nullptr;
  if (listed != nullptr) {
    tl = (listed->token_loss != nullptr) ? listed->token_loss : at<float>(workspace, lay.token_loss);
    c2 = at<float>(workspace, lay.c2);
    g_rest = at<float>(workspace, lay.g_rest);
    row_coef = at<float>(workspace, lay.row_coef);
    p_list = at<float>(workspace, lay.p_list);
    h_list = at<float>(workspace, lay.h_list);
  }

  fopd_scan_seqlens<<<1, kScanThreads, 0, s>>>(seq_lens, lag, B, T, 0, cu, flags);
  if ((st = launched()) != FOPD_OK) return st;
  const int32_t* n_use = n_train_in;
  const int32_t* nr_use = n_roll_in;
  if (n_train_in == nullptr) {
    fopd_count_train<<<B, kSegThreads, 0, s>>>(mask, cu, T, nws, nrws);
    if ((st = launched()) != FOPD_OK) return st;
    n_use = nws;
    nr_use = nrws;
  }
  if (T == 0) {      // an empty batch: loss 0, the weights of the scores, a zero projection gradient
    if (!scored) {
      fopd_segment_stats<<<B, kSegThreads, 0, s>>>(logp, behav_logp, nullptr, nullptr, teacher_logp, nullptr, mask, cu,
                                                   lag, T, hp, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                                   nullptr, nullptr, f64, nws, nrws);
      if ((st = launched()) != FOPD_OK) return st;
    }
    fopd_loss_final<<<1, kSegThreads, 0, s>>>(partials, 0, n_use, nr_use, lag, f64_use, freshness_in, B, hp.xi, loss,
                                              weights, freshness);
    if ((st = launched()) != FOPD_OK) return st;
    if (head_grad && accumulate_dweight == 0) {
      fopd_fill_zero_f32<<<static_cast<unsigned>(V), 256, 0, s>>>(dweight, lddw, static_cast<int>(d));
      return launched();
    }
    return FOPD_OK;
  }
  // the projection matrix with the vocabulary contiguous (zero beyond V), once per call
  if (grads && (st = launch_transpose(weight, ldw, V, d, Wt, ldz, ldz, s)) != FOPD_OK) return st;

  // Masked rows have no log-prob and no gradient row: each chunk's live rows are moved to the front (dense copies
  // of the per-row inputs and of the hidden rows), every kernel of the chunk runs on those, the contractions read
  // the live count on the device and leave out the tiles past it, and the per-row outputs are scattered back.  The
  // gradient side is made dense once more when the coefficients are known: rows with c_t = 0 (samples the freshness
  // weight gates out, rows outside both aligned sets' reach) get no gradient row and cost no matrix work either.
  const bool compact = (current_options().lm_head_compact != 0);
  int32_t* ex = at<int32_t>(workspace, lay.ex);
  int32_t* row_map = at<int32_t>(workspace, lay.row_map);
  int32_t* n_live = at<int32_t>(workspace, lay.n_live);
  int32_t* n_grad = n_live + 1;
  int32_t* n_chunk = n_live + 2;
  int32_t* grad_ex = at<int32_t>(workspace, lay.grad_ex);
  int64_t* cu_c = at<int64_t>(workspace, lay.cu_c);
  const float* stale = (listed != nullptr) ? listed->teacher_logp_stale : nullptr;
  // With scores supplied a chunk may cut samples anywhere, so the live rows of the whole call are numbered once and
  // chunk c is live rows c rows_chunk .. (c + 1) rows_chunk - 1: every chunk but the last is full, whatever the mask.
  // The host does not know how many there are: it walks ceil(T / rows_chunk) chunks and the last ones may be empty.
  const bool global_rows = compact && fixed;
  int32_t* keep = nullptr;             // with drop_gated: 1 for the samples of positive weight
  if (drop_gated) {
    keep = at<int32_t>(workspace, lay.keep);
    fopd_sample_keep<<<static_cast<unsigned>((B + 255) / 256), 256, 0, s>>>(nullptr, freshness_in, n_use, nr_use, lag,
                                                                          B, hp.xi, keep);
    if ((st = launched()) != FOPD_OK) return st;
  }
  if (global_rows) {
    fopd_live_scan<<<1, kLiveScanThreads, 0, s>>>(mask, nullptr, nullptr, static_cast<int>(T), cu, B, 0, ex, row_map,
                                                  n_live, cu_c, keep);
    if ((st = launched()) != FOPD_OK) return st;
  }
  if (compact && (mask != nullptr || keep != nullptr)) {
    fopd_masked_rows_zero<<<static_cast<unsigned>(T), 256, 0, s>>>(
        mask, cu, B, keep, logp, lse, tl, grads ? dhidden : nullptr, lddh, static_cast<int>(d));
    if ((st = launched()) != FOPD_OK) return st;
  }

  int64_t ci = 0;
  for (int sweep = two_sweeps ? 0 : 1; sweep < 2; ++sweep) {
  // (sweep 0, only when a sample does not fit into a chunk: logits and log-probs of every chunk, then the scores)
  ci = 0;
  for (const Chunk& c : chunks) {
    const int64_t a = c.a, R = c.R;
    if (R == 0) continue;
    const int64_t Rp = (R + 63) / 64 * 64;
    // what the chunk's kernels see: the caller's rows a .. a + R - 1, or the dense copies of the live ones
    const __bf16* Hc = Hm + a * ldh;
    int64_t ldhc = ldh;
    const int32_t* tok = token_ids + a;
    const uint8_t* msk = (mask == nullptr) ? nullptr : mask + a;
    const float* bl = behav_logp + a;
    const float* tq = (teacher_logp == nullptr) ? nullptr : teacher_logp + a;
    const int32_t* lids = (listed != nullptr) ? listed->ids + a * list_k : nullptr;
    const float* llp = (listed != nullptr) ? listed->logp + a * list_k : nullptr;
    float* lp_o = logp + a;
    float* ls_o = lse + a;
    float* tl_o = (tl != nullptr) ? tl + a : nullptr;
    float* dH = grads ? dhidden + a * lddh : nullptr;
    int64_t lddhc = lddh;
    const int64_t* cu_k = cu;           // sample offsets and the chunk's first row in the row numbering of the kernels
    int64_t a_k = a;
    const int* live = nullptr;
    // where the chunk's dense rows come from: live rows map_off .. of the numbering, as offsets from row row_base
    const int64_t map_off = global_rows ? a : 0, row_base = global_rows ? 0 : a;
    if (compact) {
      if (!global_rows) {
        fopd_live_scan<<<1, kLiveScanThreads, 0, s>>>(msk, nullptr, nullptr, static_cast<int>(R), cu, B, a, ex, row_map,
                                                      n_live, cu_c, nullptr);
        if ((st = launched()) != FOPD_OK) return st;
      }
      fopd_live_gather<<<static_cast<unsigned>(R), 256, 0, s>>>(
          row_map, n_live, map_off, row_base, n_chunk, token_ids, mask, behav_logp, teacher_logp, stale,
          (listed != nullptr) ? listed->ids : nullptr, (listed != nullptr) ? listed->logp : nullptr, list_k,
          reinterpret_cast<const uint16_t*>(Hm), ldh, static_cast<int>(d), at<int32_t>(workspace, lay.tok_c),
          at<uint8_t>(workspace, lay.mask_c), at<float>(workspace, lay.behav_c), at<float>(workspace, lay.teach_c),
          at<float>(workspace, lay.stale_c), at<int32_t>(workspace, lay.ids_c), at<float>(workspace, lay.llp_c),
          at<uint16_t>(workspace, lay.h_c));
      if ((st = launched()) != FOPD_OK) return st;
      Hc = at<__bf16>(workspace, lay.h_c);
      ldhc = d;
      tok = at<int32_t>(workspace, lay.tok_c);
      msk = at<uint8_t>(workspace, lay.mask_c);      // (never NULL from here on: the rows behind the live ones are masked)
      bl = at<float>(workspace, lay.behav_c);
      if (tq != nullptr) tq = at<float>(workspace, lay.teach_c);
      if (listed != nullptr) {
        lids = at<int32_t>(workspace, lay.ids_c);
        llp = at<float>(workspace, lay.llp_c);
        tl_o = at<float>(workspace, lay.tl_c);
      }
      lp_o = at<float>(workspace, lay.logp_c);
      ls_o = at<float>(workspace, lay.lse_c);
      if (grads) dH = at<float>(workspace, lay.dh_c);
      lddhc = d;
      cu_k = cu_c;                     // the samples' offsets in the numbering of the live rows
      a_k = map_off;
      live = n_chunk;
    }
    // the per-row outputs and dL/dhidden rows of the live rows go back to the caller's rows (the masked rows' were
    // cleared at the start)
    auto scatter = [&]() -> fopd_status {
      if (!compact) return FOPD_OK;
      fopd_live_scatter<<<static_cast<unsigned>(R), 256, 0, s>>>(
          row_map, n_live, map_off, row_base, lp_o, ls_o, tl_o, grad_ex, dH, static_cast<int>(d), logp, lse, tl,
          (grads && sweep == 1) ? dhidden : nullptr, lddh);
      return launched();
    };
    // logits of the chunk, fp32, never rounded to the storage type of stored logits
    if ((st = launch_gemm(false, Wm, ldw, V, Hc, ldhc, R, d, Z, ldz, 4, s, live)) != FOPD_OK) return st;
    if ((st = launch_k1(Z, FOPD_F32, R, V, ldz, tok, msk, lp_o, ls_o, nullptr, nullptr, flags, s)) != FOPD_OK) return st;
    if (listed != nullptr) {
      // the listed logits of each row are in the chunk's scratch: token loss, G_rest - l_t and the per-slot terms
      if ((st = launch_topk_terms(Z, FOPD_F32, R, V, ldz, tok, msk, lids, llp, list_k, listed->rest_floor, ls_o, tl_o,
                                  g_rest, p_list, h_list, s)) != FOPD_OK)
        return st;
    }
    if (sweep == 0) {
      if ((st = scatter()) != FOPD_OK) return st;
      ++ci;
      continue;
    }
    if (!fixed) {
      // the chunk holds whole samples: their scores follow from the log-probs just made
      if (compact)
        fopd_segment_stats<<<static_cast<unsigned>(c.i1 - c.i0), kSegThreads, 0, s>>>(
            lp_o, bl, nullptr, tl_o, tq, (stale != nullptr) ? at<float>(workspace, lay.stale_c) : nullptr, msk,
            cu_c + c.i0, lag + c.i0, R, hp, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
            f64 + c.i0, nws + c.i0, nrws + c.i0);
      else
        fopd_segment_stats<<<static_cast<unsigned>(c.i1 - c.i0), kSegThreads, 0, s>>>(
            logp, behav_logp, nullptr, tl, teacher_logp, stale, mask, cu + c.i0, lag + c.i0, T, hp, nullptr, nullptr,
            nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, f64 + c.i0, nws + c.i0, nrws + c.i0);
      if ((st = launched()) != FOPD_OK) return st;
    }
    const int64_t nblk = (R + kStreamThreads - 1) / kStreamThreads;
    if (listed != nullptr) {
      // c1 (into `coef`), c2 and the chunk's share of the loss; then the stream's coefficient c1 + c2 (G_rest - l_t)
      fopd_coef_loss_kl<<<static_cast<unsigned>(nblk), kStreamThreads, 0, s>>>(
          lp_o, tl_o, nullptr, bl, msk, cu_k, n_use, nr_use, lag, f64_use, freshness_in, R, B, a_k, hp, grad_scale,
          false, coef, c2, partials);
      if ((st = launched()) != FOPD_OK) return st;
      fopd_topk_row_coef<<<static_cast<unsigned>(nblk), kStreamThreads, 0, s>>>(coef, c2, g_rest, R, row_coef);
    } else {
      fopd_coef_loss<<<static_cast<unsigned>(nblk), kStreamThreads, 0, s>>>(
          lp_o, bl, tq, msk, cu_k, n_use, nr_use, lag, f64_use, freshness_in, R, B, a_k, hp, grad_scale, coef, partials,
          flags);
    }
    if ((st = launched()) != FOPD_OK) return st;
    // (weights and scores of samples whose chunk is still to come are overwritten by the later calls)
    fopd_loss_final<<<1, kSegThreads, 0, s>>>(partials, nblk, n_use, nr_use, lag, f64_use, freshness_in, B, hp.xi,
                                              chunk_loss + ci, weights, freshness);
    if ((st = launched()) != FOPD_OK) return st;
    if (!grads) {
      if ((st = scatter()) != FOPD_OK) return st;
      ++ci;
      continue;
    }
    const int32_t* gex = nullptr;        // the rows that have a gradient row, counted among the chunk's (live) rows
    const __bf16* Hg = Hc;               // their hidden rows
    int64_t rows_hg = R;
    if (compact) {
      fopd_live_scan<<<1, kLiveScanThreads, 0, s>>>(nullptr, coef, (listed != nullptr) ? c2 : nullptr,
                                                    static_cast<int>(R), nullptr, -1, 0, grad_ex, nullptr, n_grad,
                                                    nullptr, nullptr);
      if ((st = launched()) != FOPD_OK) return st;
      fopd_grad_gather<<<static_cast<unsigned>(R), 256, 0, s>>>(grad_ex, reinterpret_cast<const uint16_t*>(Hc), ldhc,
                                                               static_cast<int>(d), at<uint16_t>(workspace, lay.h_g));
      if ((st = launched()) != FOPD_OK) return st;
      gex = grad_ex;
      Hg = at<__bf16>(workspace, lay.h_g);
      rows_hg = Rp;
      live = n_grad;
    }
    {
      ScopedTimer timer(1, s);
      fopd_k4_grad_wide<<<static_cast<unsigned>(R), kGradThreads, 0, s>>>(
          Z, ldz, reinterpret_cast<uint16_t*>(G), ldz, static_cast<int>(V), tok, ls_o, lp_o,
          (listed != nullptr) ? row_coef : coef, gex);
      if ((st = launched()) != FOPD_OK) return st;
      if (listed != nullptr) {
        // the k listed entries of each row and the sampled token's, in the bf16 rows just written
        const dim3 grid(static_cast<unsigned>((R + kListRows - 1) / kListRows)), block(kListThreads);
        fopd_topk_fixup<FOPD_BF16><<<grid, block, 0, s>>>(G, R, static_cast<int>(V), ldz, tok, lids, list_k, lp_o, coef,
                                                         c2, g_rest, p_list, h_list, gex);
        if ((st = launched()) != FOPD_OK) return st;
      }
    }
    // the contraction over rows reads whole steps of 64 rows: zeros behind the last gradient row
    if (compact) {
      fopd_grad_tail_zero<<<64, 256, 0, s>>>(n_grad, reinterpret_cast<uint16_t*>(G), ldz,
                                             at<uint16_t>(workspace, lay.h_g), static_cast<int>(d));
      if ((st = launched()) != FOPD_OK) return st;
    } else if (Rp > R) {
      fopd_fill_zero_f32<<<static_cast<unsigned>(Rp - R), 256, 0, s>>>(reinterpret_cast<float*>(G + R * ldz), ldz / 2,
                                                                     static_cast<int>(ldz / 2));
      if ((st = launched()) != FOPD_OK) return st;
    }
    // dL/dhidden of the chunk: rows x hidden, contraction over the vocabulary
    if ((st = launch_gemm(false, Wt, ldz, d, G, ldz, R, ldz, dH, lddhc, 5, s, live)) != FOPD_OK) return st;
    // dL/dweight: vocabulary x hidden, contraction over the chunk's rows, both operands as they are stored
    const bool acc = (ci > 0) || (accumulate_dweight != 0);
    if (head_grad &&
        (st = launch_gemm_tn(acc, Hg, compact ? d : ldhc, d, rows_hg, G, ldz, V, Rp, dweight, lddw, 6, s, live)) != FOPD_OK)
      return st;
    if ((st = scatter()) != FOPD_OK) return st;
    ++ci;
  }
  if (sweep == 0) {
    // every sample's log-probs (and token losses) are in the caller's arrays: the scores of all samples at once
    fopd_segment_stats<<<static_cast<unsigned>(B), kSegThreads, 0, s>>>(
        logp, behav_logp, nullptr, tl, teacher_logp, stale, mask, cu, lag, T, hp, nullptr, nullptr, nullptr, nullptr,
        nullptr, nullptr, nullptr, nullptr, f64, nws, nrws);
    if ((st = launched()) != FOPD_OK) return st;
    if (global_rows) {
      // the log-probs of every live row are in place: the second sweep leaves the samples of weight 0 out altogether
      keep = at<int32_t>(workspace, lay.keep);
      fopd_sample_keep<<<static_cast<unsigned>((B + 255) / 256), 256, 0, s>>>(f64, nullptr, n_use, nr_use, lag, B, hp.xi,
                                                                            keep);
      if ((st = launched()) != FOPD_OK) return st;
      fopd_live_scan<<<1, kLiveScanThreads, 0, s>>>(mask, nullptr, nullptr, static_cast<int>(T), cu, B, 0, ex, row_map,
                                                    n_live, cu_c, keep);
      if ((st = launched()) != FOPD_OK) return st;
      if (grads) {
        fopd_masked_rows_zero<<<static_cast<unsigned>(T), 256, 0, s>>>(mask, cu, B, keep, nullptr, nullptr, nullptr,
                                                                       dhidden, lddh, static_cast<int>(d));
        if ((st = launched()) != FOPD_OK) return st;
      }
    }
  }
  }
  fopd_sum_chunks<<<1, 64, 0, s>>>(chunk_loss, static_cast<int>(ci), loss);
  return launched();
}

fopd_status fopd_lm_head_loss_fwd_bwd(const void* hidden, int64_t ldh, const void* weight, int64_t ldw, int64_t T,
                                      int64_t V, int64_t d, const int32_t* token_ids, const uint8_t* mask,
                                      const float* behav_logp, const float* teacher_logp, const int32_t* seq_lens,
                                      const int32_t* lag, int32_t B, fopd_hparams hp, const float* freshness_in,
                                      const int32_t* n_train_in, const int32_t* n_roll_in,
                                      const int32_t* seq_lens_host, float grad_scale, int64_t rows_chunk, float* loss,
                                      float* freshness, float* weights, float* logp, float* lse, float* dhidden,
                                      int64_t lddh, float* dweight, int64_t lddw, int accumulate_dweight,
                                      void* workspace, size_t workspace_bytes, void* stream) {
  return lm_head_loss_impl(hidden, ldh, weight, ldw, T, V, d, token_ids, mask, behav_logp, teacher_logp, seq_lens, lag,
                           B, hp, freshness_in, n_train_in, n_roll_in, seq_lens_host, grad_scale, rows_chunk, loss,
                           freshness, weights, logp, lse, dhidden, lddh, dweight, lddw, accumulate_dweight, nullptr,
                           workspace, workspace_bytes, stream);
}

size_t fopd_lm_head_loss_topk_workspace_bytes(int64_t T, int64_t V, int64_t d, int32_t B, int64_t rows_chunk,
                                              int32_t k) {
  return LmLossWorkspace(T, V, d, B, rows_chunk, k < 1 ? 1 : k).total;
}

fopd_status fopd_lm_head_loss_fwd_bwd_topk_teacher(
    const void* hidden, int64_t ldh, const void* weight, int64_t ldw, int64_t T, int64_t V, int64_t d,
    const int32_t* token_ids, const uint8_t* mask, const float* behav_logp, const int32_t* list_ids,
    const float* list_logp, int32_t k, float rest_floor, const float* teacher_logp, const float* teacher_logp_stale,
    const int32_t* seq_lens, const int32_t* lag, int32_t B, fopd_hparams hp, const float* freshness_in,
    const int32_t* n_train_in, const int32_t* n_roll_in, const int32_t* seq_lens_host, float grad_scale,
    int64_t rows_chunk, float* loss, float* freshness, float* weights, float* logp, float* lse, float* token_loss,
    float* dhidden, int64_t lddh, float* dweight, int64_t lddw, int accumulate_dweight, void* workspace,
    size_t workspace_bytes, void* stream) {
  ListedTeacher listed;
  listed.ids = list_ids;
  listed.logp = list_logp;
  listed.k = k;
  listed.rest_floor = rest_floor;
  listed.teacher_logp_stale = teacher_logp_stale;
  listed.token_loss = token_loss;
  return lm_head_loss_impl(hidden, ldh, weight, ldw, T, V, d, token_ids, mask, behav_logp, teacher_logp, seq_lens, lag,
                           B, hp, freshness_in, n_train_in, n_roll_in, seq_lens_host, grad_scale, rows_chunk, loss, freshness,
                           weights, logp, lse, dhidden, lddh, dweight, lddw, accumulate_dweight, &listed, workspace,
                           workspace_bytes, stream);
}

fopd_status fopd_set_option(const char* name, int value) {
  if (name == nullptr) return FOPD_EINVAL;
  const std::string key(name);
  std::lock_guard<std::mutex> lock(g_state_mutex);
  if (key == "k14_threads") {
    if (value != 256 && value != 512 && value != 1024) return FOPD_EINVAL;
    g_opt.k14_threads = value;
    return FOPD_OK;
  }
  if (key == "k14_regs") {
    if (value != 0 && value != 1) return FOPD_EINVAL;
    g_opt.k14_regs = value;
    return FOPD_OK;
  }
  if (key == "k14_regs_grid") {
    if (value < 0 || value > 4096) return FOPD_EINVAL;
    g_opt.k14_regs_grid = value;
    return FOPD_OK;
  }
  if (key == "k4_regs") {
    if (value != 0 && value != 1) return FOPD_EINVAL;
    g_opt.k4_regs = value;
    return FOPD_OK;
  }
  if (key == "lm_head_compact") {
    if (value != 0 && value != 1) return FOPD_EINVAL;
    g_opt.lm_head_compact = value;
    return FOPD_OK;
  }
  if (key == "k14_rows_per_cu") {
    if (value < 1 || value > 8) return FOPD_EINVAL;
    g_opt.k14_rows_per_cu = value;
    return FOPD_OK;
  }
  return FOPD_EINVAL;
}

fopd_status fopd_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_state_mutex);
  g_prof.on = (on != 0);
  return FOPD_OK;
}

fopd_status fopd_profile_reset(void) {
  std::lock_guard<std::mutex> lock(g_state_mutex);
  for (int i = 0; i < kProfSlots; ++i) g_prof.used[i] = 0;
  return FOPD_OK;
}

fopd_status fopd_profile_read(int which, double* total_ms_host, int64_t* launches_host) {
  if (which < 0 || which >= kProfSlots || total_ms_host == nullptr || launches_host == nullptr) return FOPD_EINVAL;
  std::vector<hipEvent_t> start, stop;
  {
    std::lock_guard<std::mutex> lock(g_state_mutex);
    start.assign(g_prof.start[which].begin(), g_prof.start[which].begin() + g_prof.used[which]);
    stop.assign(g_prof.stop[which].begin(), g_prof.stop[which].begin() + g_prof.used[which]);
  }
  double tot = 0.0;
  for (size_t i = 0; i < start.size(); ++i) {
    if (hipEventSynchronize(stop[i]) != hipSuccess) return FOPD_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, start[i], stop[i]) != hipSuccess) return FOPD_EHIP;
    tot += ms;
  }
  *total_ms_host = tot;
  *launches_host = static_cast<int64_t>(start.size());
  return FOPD_OK;
}

}  // extern "C"
