// HIP kernels of the f-OPD loss pass for gfx950 (CDNA4, 64-wide wavefronts).
//
// Two kernels stream the [T, V] logits and are bound by HBM bandwidth:
//   fopd_k1_lse   one read of the logits  -> lse_t, lp_t            (Eq. "kl-diagnostics" /
//                                                                     Eq. "sample-aggregated-loss": pi_theta^t(y|x))
//   fopd_k4_grad  one read + one write    -> c_t (softmax - onehot)  (gradient of Algorithm 1's anchored loss)
// The remaining kernels touch only O(T) + O(B) data:
//   fopd_scan_seqlens   segment offsets, argument checks
//   fopd_segment_stats  per-sample D^roll, D^sup, l_i, coverage, freshness (Eq. "freshness")
//   fopd_aggregate      buffer means of Sec. 4.2
//   fopd_coef_loss      per-token gradient coefficient and loss partial sums
//   fopd_loss_final     loss scalar and weights
// A third streaming kernel, fopd_k14_fused, does both passes over a row in one workgroup when the
// freshness scores are supplied by the caller (second loop of Algorithm 1 on its own).
// fopd_k5_kl / fopd_coef_loss_kl / fopd_k6_grad_kl are the same two passes over two logits tensors: the
// second is either the stale checkpoint's (full-vocabulary rollout drift) or the teacher's
// (distribution-level token loss).
//
// There is no matrix contraction anywhere on this path, so no MFMA is used.  All reductions
// run in a fixed order (wavefront shuffles, then LDS), so results are bit-reproducible.

#ifndef FOPD_KERNELS_HIP_
#define FOPD_KERNELS_HIP_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fopd.h"

namespace fopd {

constexpr int kStreamThreads = 256;   // 4 wavefronts per row in the streaming kernels
constexpr int kGradThreads = 256;     // the gradient kernel: 64..512 lanes and 2..8 loads in flight were
constexpr int kGradUnroll = 2;        // A/B-tested in one process; all within 1 %, this pair the fastest
constexpr int kUnroll = 4;            // 16-byte loads in flight per lane and loop trip
constexpr int kScanThreads = 1024;
constexpr int kSegThreads = 512;
enum : int32_t { kFlagToken = 1, kFlagSegments = 2, kFlagLag = 4, kFlagSets = 8 };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr float kLog2e = 1.4426950408889634f;   // nearest float to log2(e)
constexpr double kLn2 = 0.6931471805599453094;

template <int DT> struct Elem;
template <> struct Elem<FOPD_F32> {
  static constexpr int kPerVec = 4;
  static constexpr int kBytes = 4;
};
template <> struct Elem<FOPD_BF16> {
  static constexpr int kPerVec = 8;
  static constexpr int kBytes = 2;
};

// ---- element access -------------------------------------------------------------------

template <int DT>
__device__ __forceinline__ void unpack(const u32x4& q, float* x);

template <>
__device__ __forceinline__ void unpack<FOPD_F32>(const u32x4& q, float* x) {
  x[0] = __uint_as_float(q.x);
  x[1] = __uint_as_float(q.y);
  x[2] = __uint_as_float(q.z);
  x[3] = __uint_as_float(q.w);
}

// A bf16 is the upper half of a float: element 2k sits in the low half of word k.
template <>
__device__ __forceinline__ void unpack<FOPD_BF16>(const u32x4& q, float* x) {
  x[0] = __uint_as_float(q.x << 16);
  x[1] = __uint_as_float(q.x & 0xffff0000u);
  x[2] = __uint_as_float(q.y << 16);
  x[3] = __uint_as_float(q.y & 0xffff0000u);
  x[4] = __uint_as_float(q.z << 16);
  x[5] = __uint_as_float(q.z & 0xffff0000u);
  x[6] = __uint_as_float(q.w << 16);
  x[7] = __uint_as_float(q.w & 0xffff0000u);
}

template <int DT>
__device__ __forceinline__ float load_elem(const void* row, int idx);
template <>
__device__ __forceinline__ float load_elem<FOPD_F32>(const void* row, int idx) {
  return static_cast<const float*>(row)[idx];
}
template <>
__device__ __forceinline__ float load_elem<FOPD_BF16>(const void* row, int idx) {
  return __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t*>(row)[idx]) << 16);
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two floats -> two bf16 in one word, round to nearest even (gfx950 has a packed convert).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, b);
}

template <int DT>
__device__ __forceinline__ u32x4 pack(const float* g);
template <>
__device__ __forceinline__ u32x4 pack<FOPD_F32>(const float* g) {
  return u32x4{__float_as_uint(g[0]), __float_as_uint(g[1]), __float_as_uint(g[2]),
                    __float_as_uint(g[3])};
}
template <>
__device__ __forceinline__ u32x4 pack<FOPD_BF16>(const float* g) {
  return u32x4{pack_bf16x2(g[0], g[1]), pack_bf16x2(g[2], g[3]), pack_bf16x2(g[4], g[5]),
                    pack_bf16x2(g[6], g[7])};
}

template <int DT>
__device__ __forceinline__ void store_elem(void* row, int idx, float g);
template <>
__device__ __forceinline__ void store_elem<FOPD_F32>(void* row, int idx, float g) {
  static_cast<float*>(row)[idx] = g;
}
template <>
__device__ __forceinline__ void store_elem<FOPD_BF16>(void* row, int idx, float g) {
  static_cast<uint16_t*>(row)[idx] = static_cast<uint16_t>(pack_bf16x2(g, 0.0f) & 0xffffu);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- wavefront / block reductions (fixed order) ----------------------------------------

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Sum over a block of NT threads; the result is valid in thread 0.  `sh` holds NT/64 doubles.
template <int NT>
__device__ __forceinline__ double block_sum(double v, double* sh) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[w] = v;
  __syncthreads();
  double tot = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) tot += sh[i];
  }
  return tot;
}

// ---- online log-sum-exp state of one lane ----------------------------------------------
// The lane holds rL (its running maximum times log2 e, as rounded) and s = sum 2^t over the
// elements it has seen, t = x log2e - rL, the sampled token excluded; with ENT also w = sum t 2^t,
// from which the row's entropy follows without cancellation at the scale of the logits
// (monitoring proxy, App. B "response entropy").

struct LaneState {
  float r = -1.0e38f;                       // "nothing seen yet" (finite on purpose)
  float rL = -1.0e38f * 1.4426950408889634f;
  float s = 0.f;
  float w = 0.f;
};

// Moves a (s, w) pair from reference `from` to reference `to` (both in log2 units).
__device__ __forceinline__ void rebase(float from, float to, float& s, float& w, bool ent) {
  const float scale = fast_exp2(from - to);
  if (ent) w = fmaf(from - to, s, w) * scale;
  s *= scale;
}

// max(x, -1e30) as one integer instruction: among floats with the sign bit set the bit pattern grows with the
// magnitude, and every pattern without the sign bit is smaller, so an unsigned minimum with the pattern of -1e30
// replaces exactly the values below it (-inf included).  fmaxf costs two instructions here (the canonicalisation
// of its operand that IEEE maximum semantics ask for comes first).
__device__ __forceinline__ float floor_minus_inf(float x) {
  const uint32_t kFloorBits = 0xf149f2cau;             // -1e30f
  return __uint_as_float(min(__float_as_uint(x), kFloorBits));
}

template <int N, bool ENT>
__device__ __forceinline__ void accumulate(const float* x, LaneState& st) {
  // The maximum starts from the running one, so that every step is a three-operand maximum of the chain and two
  // entries (a two-operand first step costs two extra instructions: hipcc canonicalises both of its operands).
  float bm = st.r;
#pragma unroll
  for (int i = 0; i < N; ++i) bm = fmaxf(bm, x[i]);
  if (bm > st.r) {                    // rare after the first few vectors
    const float nrL = bm * kLog2e;
    rebase(st.rL, nrL, st.s, st.w, ENT);
    st.r = bm;
    st.rL = nrL;
  }
  // two chains per sum, started by the first two entries (no additions to zero)
  float a0 = 0.f, a1 = 0.f, w0 = 0.f, w1 = 0.f;
#pragma unroll
  for (int i = 0; i < N; i += 2) {
    const float t0 = fmaf(x[i], kLog2e, -st.rL);
    const float e0 = fast_exp2(t0);
    a0 = (i == 0) ? e0 : a0 + e0;
    if (ENT) w0 = (i == 0) ? e0 * floor_minus_inf(t0) : fmaf(e0, floor_minus_inf(t0), w0);   // t = -inf has e = 0: keep 0 * t finite
    if (i + 1 < N) {
      const float t1 = fmaf(x[i + 1], kLog2e, -st.rL);
      const float e1 = fast_exp2(t1);
      a1 = (i == 0) ? e1 : a1 + e1;
      if (ENT) w1 = (i == 0) ? e1 * floor_minus_inf(t1) : fmaf(e1, floor_minus_inf(t1), w1);
    }
  }
  st.s += a0 + a1;
  if (ENT) st.w += w0 + w1;
}

// ---- row routines shared by the streaming kernels ----------------------------------------
// NT lanes walk one row of V elements in 16-byte vectors, U vectors in flight per lane and trip;
// vector j of a trip belongs to lane j % NT, so a wavefront instruction touches 1 KB contiguous.
// CACHED selects ordinary loads (lines stay in L2 / Infinity Cache for a second pass over the
// same row) instead of non-temporal ones.

template <bool CACHED>
__device__ __forceinline__ u32x4 load_vec(const u32x4* p) {
  if (CACHED) return *p;
  return __builtin_nontemporal_load(p);
}

// Pass over a row for the log-sum-exp: updates the lane's state; the lane that meets the
// sampled token y stores its value to *zy_out (LDS) and leaves it out of the sum.
template <int DT, int NT, int U, bool CACHED, bool ENT>
__device__ __forceinline__ void row_lse(const char* row, int V, int y, LaneState& st, float* zy_out) {
  constexpr int E = Elem<DT>::kPerVec;
  const u32x4* rv = reinterpret_cast<const u32x4*>(row);
  const int tid = threadIdx.x;
  const int nvec = V / E;
  const int jy = y / E, ey = y % E;
  const float kNegInf = -__builtin_inff();
  // the sampled token sits in exactly one trip of the loop: a wavefront-uniform test keeps the
  // per-vector comparisons out of all the others
  const int ytrip = jy / (U * NT);
  int trip = 0;
  int j = tid;
  for (; j + (U - 1) * NT < nvec; j += U * NT, ++trip) {
    u32x4 q[U];
#pragma unroll
    for (int u = 0; u < U; ++u) q[u] = load_vec<CACHED>(rv + j + u * NT);
    float x[U * E];
#pragma unroll
    for (int u = 0; u < U; ++u) unpack<DT>(q[u], x + u * E);
    if (trip == ytrip) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (j + u * NT == jy) {
#pragma unroll
          for (int e = 0; e < E; ++e) {
            if (e == ey) {
              *zy_out = x[u * E + e];
              x[u * E + e] = kNegInf;
            }
          }
        }
      }
    }
    accumulate<U * E, ENT>(x, st);
  }
  for (; j < nvec; j += NT) {
    const u32x4 q = load_vec<CACHED>(rv + j);
    float x[E];
    unpack<DT>(q, x);
    if (j == jy) {
#pragma unroll
      for (int e = 0; e < E; ++e) {
        if (e == ey) {
          *zy_out = x[e];
          x[e] = kNegInf;
        }
      }
    }
    accumulate<E, ENT>(x, st);
  }
  {
    const int idx = nvec * E + tid;   // ragged tail: fewer than E elements
    if (idx < V) {
      float x1 = load_elem<DT>(row, idx);
      if (idx == y) {
        *zy_out = x1;
        x1 = kNegInf;
      }
      accumulate<1, ENT>(&x1, st);
    }
  }
}

// Thread 0's part of the row's finish: merges the n_waves (reference, sum) pairs that the wavefronts left in
// sh_R / sh_S (and the entropy sums in sh_W with ENT) and forms lp, lse (and the row entropy) in fp64.
template <bool ENT>
__device__ __forceinline__ void lse_from_partials(const float* zy_in, const float* sh_R, const float* sh_S,
                                                  const float* sh_W, int n_waves, double& lp_out, double& lse_out,
                                                  double& ent_out) {
  float RR = sh_R[0];
  for (int i = 1; i < n_waves; ++i) RR = fmaxf(RR, sh_R[i]);
  float SS = 0.f, WW = 0.f;
  for (int i = 0; i < n_waves; ++i) {
    float si = sh_S[i], wi = ENT ? sh_W[i] : 0.f;
    rebase(sh_R[i], RR, si, wi, ENT);
    SS += si;
    WW += wi;
  }
  // Everything below is in log2 units of the scaled logits x * kLog2e.
  //   a2 = log2( sum_{v != y} 2^(x_v) / 2^(x_y) )   log-odds of "not y"
  //   lp = -log(1 + 2^a2),  lse = x_y + log(1 + 2^a2)
  const double zyL = static_cast<double>(*zy_in) * static_cast<double>(kLog2e);
  const double others = static_cast<double>(RR) + log2(static_cast<double>(SS));   // log2 sum_{v != y}
  const double a2 = others - zyL;
  const double q = exp2(-fabs(a2));                  // 2^-|a2|, in (0, 1]
  const double l1q = log1p(q) * (1.0 / kLn2);        // log2(1 + 2^-|a2|)
  const double sp = (a2 > 0.0 ? a2 : 0.0) + l1q;
  lp_out = -sp * kLn2;
  // the larger of the two parts plus the correction: stays finite when z_y = -inf (lp = -inf) or when
  // every other logit is -inf (lp = 0)
  lse_out = ((a2 > 0.0 ? others : zyL) + l1q) * kLn2;
  ent_out = 0.0;
  if (ENT) {
    // H = h(p_y) + (1 - p_y) * H(softmax over the other tokens): the binary entropy of
    // {y, not y} plus the conditional entropy, each a sum of non-negative terms.
    const double a = fabs(a2);
    const double h2 = (a < 1.0e300) ? l1q + a * q / (1.0 + q) : 0.0;
    const double p_not = (a2 > 0.0) ? 1.0 / (1.0 + q) : q / (1.0 + q);
    double h_ex = 0.0;
    if (SS > 0.f) h_ex = log2(static_cast<double>(SS)) - static_cast<double>(WW) / static_cast<double>(SS);
    if (h_ex < 0.0) h_ex = 0.0;
    ent_out = (h2 + p_not * h_ex) * kLn2;
  }
}

// The wavefronts' part: a common reference per wavefront, then its (reference, sum) pair into sh_R / sh_S
// (sh_W with ENT), NT/64 floats each.  Ends with the one __syncthreads of the finish.
template <int NT, bool ENT>
__device__ __forceinline__ void block_lse_merge(const LaneState& st, float* sh_R, float* sh_S, float* sh_W) {
  const float Rw = wave_max(st.rL);
  float ls = st.s, lw = st.w;
  rebase(st.rL, Rw, ls, lw, ENT);
  const float Sw = wave_sum(ls);
  float Ww = 0.f;
  if (ENT) Ww = wave_sum(lw);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) {
    sh_R[w] = Rw;
    sh_S[w] = Sw;
    if (ENT) sh_W[w] = Ww;
  }
  __syncthreads();
}

// Merges the lanes' states; thread 0 returns lp, lse (and with ENT the row entropy) in fp64, the
// other lanes return zeros.  Contains one __syncthreads.  sh_R / sh_S / sh_W hold NT/64 floats each.
template <int NT, bool ENT>
__device__ __forceinline__ void block_lse_finish(const LaneState& st, const float* zy_in, float* sh_R,
                                                 float* sh_S, float* sh_W, double& lp_out, double& lse_out,
                                                 double& ent_out) {
  block_lse_merge<NT, ENT>(st, sh_R, sh_S, sh_W);
  lp_out = 0.0;
  lse_out = 0.0;
  ent_out = 0.0;
  if (threadIdx.x == 0) lse_from_partials<ENT>(zy_in, sh_R, sh_S, sh_W, NT / 64, lp_out, lse_out, ent_out);
}

// Gradient row: g_v = c * 2^(x_v log2e - lseL), the sampled token's entry replaced by gy.
// Input and output rows may be the same memory: each vector is read and written by one lane.
template <int DT, int NT, int U, bool CACHED>
__device__ __forceinline__ void row_grad(const char* row, char* orow, int V, int y, float c, float lseL,
                                         float gy) {
  constexpr int E = Elem<DT>::kPerVec;
  const u32x4* rv = reinterpret_cast<const u32x4*>(row);
  u32x4* ov = reinterpret_cast<u32x4*>(orow);
  const int tid = threadIdx.x;
  const int nvec = V / E;
  const int jy = y / E, ey = y % E;
  // the sampled token sits in exactly one trip of the loop: a wavefront-uniform test keeps the
  // per-vector comparisons out of all the others
  const int ytrip = jy / (U * NT);
  int trip = 0;
  int j = tid;
  for (; j + (U - 1) * NT < nvec; j += U * NT, ++trip) {
    u32x4 q[U];
#pragma unroll
    for (int u = 0; u < U; ++u) q[u] = load_vec<CACHED>(rv + j + u * NT);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[E];
      unpack<DT>(q[u], x);
#pragma unroll
      for (int e = 0; e < E; ++e) x[e] = c * fast_exp2(fmaf(x[e], kLog2e, -lseL));
      if (trip == ytrip && j + u * NT == jy) {
#pragma unroll
        for (int e = 0; e < E; ++e)
          if (e == ey) x[e] = gy;
      }
      __builtin_nontemporal_store(pack<DT>(x), ov + j + u * NT);
    }
  }
  for (; j < nvec; j += NT) {
    const u32x4 q = load_vec<CACHED>(rv + j);
    float x[E];
    unpack<DT>(q, x);
#pragma unroll
    for (int e = 0; e < E; ++e) x[e] = c * fast_exp2(fmaf(x[e], kLog2e, -lseL));
    if (j == jy) {
#pragma unroll
      for (int e = 0; e < E; ++e)
        if (e == ey) x[e] = gy;
    }
    __builtin_nontemporal_store(pack<DT>(x), ov + j);
  }
  {
    const int idx = nvec * E + tid;
    if (idx < V) {
      float g = c * fast_exp2(fmaf(load_elem<DT>(row, idx), kLog2e, -lseL));
      if (idx == y) g = gy;
      store_elem<DT>(orow, idx, g);
    }
  }
}

template <int DT, int NT>
__device__ __forceinline__ void row_zero(char* orow, int V) {
  constexpr int E = Elem<DT>::kPerVec;
  u32x4* ov = reinterpret_cast<u32x4*>(orow);
  const int nvec = V / E;
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  for (int j = threadIdx.x; j < nvec; j += NT) __builtin_nontemporal_store(zero, ov + j);
  const int idx = nvec * E + threadIdx.x;
  if (idx < V) store_elem<DT>(orow, idx, 0.f);
}

// e^d * d - e^d + 1 without cancellation for small d
__device__ __forceinline__ double kl_term(double d, double* rho_out) {
  const double e1 = expm1(d);
  if (rho_out != nullptr) *rho_out = e1 + 1.0;
  return d * e1 + (d - e1);
}

// The two aligned sets of Sec. 4.1 in one byte per row: 0 = in neither, 2 = in U^roll only,
// 3 = in U^sup only, anything else (a plain loss mask's 1) = in both.  No mask = all rows in both.
__device__ __forceinline__ bool in_sup_set(const uint8_t* mask, int64_t t) {
  if (mask == nullptr) return true;
  const uint8_t m = mask[t];
  return m != 0 && m != 2;
}
__device__ __forceinline__ bool in_roll_set(const uint8_t* mask, int64_t t) {
  if (mask == nullptr) return true;
  const uint8_t m = mask[t];
  return m != 0 && m != 3;
}

// A row that is in exactly one of the two sets (mask byte 2 or 3).
__device__ __forceinline__ bool in_one_set_only(const uint8_t* mask, int64_t t) {
  return mask != nullptr && (mask[t] == 2 || mask[t] == 3);
}

// ReLU(f - xi); 0 for an invalid sample (either aligned set empty, or a negative lag, which is also
// flagged), whatever xi is.
__device__ __forceinline__ double weight_of(double f, int32_t n_sup, int32_t n_roll, int32_t lag, float xi) {
  if (n_sup <= 0 || n_roll <= 0 || lag < 0) return 0.0;
  const double w = f - static_cast<double>(xi);
  return w > 0.0 ? w : 0.0;
}

// The weight of the kernels that make both passes over a row: from the supplied scores, or, when there are none
// (fresh32 == nullptr: the gradient rows are wanted at unit sample weight), 1 for a valid sample and 0 otherwise.
__device__ __forceinline__ double row_pass_weight(const float* fresh32, int i, int32_t n_sup, int32_t n_roll,
                                                  int32_t lag, float xi) {
  if (fresh32 == nullptr) return (n_sup <= 0 || n_roll <= 0 || lag < 0) ? 0.0 : 1.0;
  return weight_of(static_cast<double>(fresh32[i]), n_sup, n_roll, lag, xi);
}

// Row coefficient c_t and the row's share of the loss, from the fp32-rounded log-prob:
//   c_t = g w / B ( [t in U^sup] (lq - lp) / |U^sup|  -  [t in U^roll] lambda rho d / |U^roll| ).
__device__ __forceinline__ float coef_and_loss(double lp, double lb, double lq, double w, int32_t n_sup,
                                               int32_t n_roll, bool sup, bool roll, int32_t B, fopd_hparams hp,
                                               float grad_scale, double* loss_term) {
  const double wb = w / static_cast<double>(B);
  const double lam = hp.lambda;
  double lt = 0.0, c = 0.0;
  if (sup) {
    lt += (lp - lq) / static_cast<double>(n_sup);
    c += (lq - lp) / static_cast<double>(n_sup);
  }
  if (roll) {
    double rho;
    const double d = lp - lb;
    const double k = kl_term(d, &rho);
    lt += lam * k / static_cast<double>(n_roll);
    c -= lam * rho * d / static_cast<double>(n_roll);
  }
  *loss_term = wb * lt;
  return static_cast<float>(static_cast<double>(grad_scale) * wb * c);
}

// Largest i with cu[i] <= gt, given cu[0] <= gt < cu[B].
__device__ __forceinline__ int sample_of_row(const int64_t* cu, int32_t B, int64_t gt) {
  int lo = 0, hi = B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= gt) lo = mid; else hi = mid;
  }
  return lo;
}

}  // namespace

// =========================================================================================
// K1: streaming log-sum-exp and sampled-token log-probability.  One workgroup per row.
// =========================================================================================

template <int DT, int U, bool ENT>
__global__ void __launch_bounds__(kStreamThreads)
fopd_k1_lse(const void* logits, int64_t T, int V, int64_t ld, const int32_t* token_ids,
            const uint8_t* mask, float* logp, float* lse, int64_t* gather_idx, float* entropy,
            int32_t* flags) {
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x;
  const int y = token_ids[t];
  if (tid == 0 && gather_idx != nullptr) gather_idx[t] = t * ld + static_cast<int64_t>(y);
  bool live = (mask == nullptr) || (mask[t] != 0);
  if (live && (y < 0 || y >= V)) {
    if (tid == 0) atomicOr(flags, kFlagToken);
    live = false;
  }
  if (!live) {
    if (tid == 0) {
      logp[t] = 0.f;
      lse[t] = 0.f;
      if (ENT) entropy[t] = 0.f;
    }
    return;
  }
  __shared__ float sh_zy;
  __shared__ float sh_R[kStreamThreads / 64];
  __shared__ float sh_S[kStreamThreads / 64];
  __shared__ float sh_W[kStreamThreads / 64];
  const char* row = static_cast<const char*>(logits) + t * ld * Elem<DT>::kBytes;
  LaneState st;
  row_lse<DT, kStreamThreads, U, false, ENT>(row, V, y, st, &sh_zy);
  double lp, ls, ent;
  block_lse_finish<kStreamThreads, ENT>(st, &sh_zy, sh_R, sh_S, sh_W, lp, ls, ent);
  if (tid == 0) {
    logp[t] = static_cast<float>(lp);
    lse[t] = static_cast<float>(ls);
    if (ENT) entropy[t] = static_cast<float>(ent);
  }
}

// =========================================================================================
// K4: gradient stream.  dlogits[t, v] = c_t * (exp(z - lse_t) - [v == y_t]).  One workgroup
// per row; rows with c_t == 0 are zero-filled without reading the logits.  `dlogits` may be
// the same buffer as `logits`: every 16-byte vector is read and written by the same lane.
// =========================================================================================

template <int DT, int U>
__global__ void __launch_bounds__(kGradThreads)
fopd_k4_grad(const void* logits, void* dlogits, int64_t T, int V, int64_t ld,
             const int32_t* token_ids, const float* lse, const float* logp, const float* coef) {
  const int64_t t = blockIdx.x;
  const float c = coef[t];
  const int y = token_ids[t];
  char* orow = static_cast<char*>(dlogits) + t * ld * Elem<DT>::kBytes;
  if (c == 0.f || y < 0 || y >= V) {     // a token id out of range was flagged by the first pass: no gradient
    row_zero<DT, kGradThreads>(orow, V);
    return;
  }
  const char* row = static_cast<const char*>(logits) + t * ld * Elem<DT>::kBytes;
  // the sampled token's entry c * (p_y - 1) comes from lp_y, which stays accurate as p_y -> 1
  row_grad<DT, kGradThreads, U, false>(row, orow, V, y, c, lse[t] * kLog2e, c * expm1f(logp[t]));
}

// =========================================================================================
// K14: both passes over one row in one workgroup, for calls whose freshness scores are given.
// The first pass uses ordinary loads so that the row stays in the Infinity Cache; the second
// pass re-reads it from there and writes the gradient: HBM sees one read and one write per
// row.  NT lanes per row; the caller caps the rows in flight per compute unit through the
// dynamic LDS size (launch shapes measured on MI355X: 256 lanes x 6 rows is the fastest).
// With NT = kStreamThreads it produces the same bits as K1 + fopd_coef_loss + K4 (same partition of
// the row over lanes); other NT sum the row in another order and may differ in the last place.
// =========================================================================================

template <int DT, int NT, int U>
__global__ void __launch_bounds__(NT)
fopd_k14_fused(const void* logits, void* dlogits, int64_t T, int V, int64_t ld, const int32_t* token_ids,
               const uint8_t* mask, const float* behav_logp, const float* teacher_logp, const int64_t* cu,
               const int32_t* n_train, const int32_t* n_roll, const int32_t* lag, const float* fresh32, int32_t B,
               int64_t row_begin, fopd_hparams hp, float grad_scale, float* logp, double* row_loss, int32_t* flags) {
  extern __shared__ char occupancy_pad[];      // sized by the host only to cap workgroups per CU
  __shared__ float sh_zy;
  __shared__ float sh_R[NT / 64];
  __shared__ float sh_S[NT / 64];
  __shared__ float sh_c, sh_lseL, sh_gy;
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x;
  const int y = token_ids[t];
  char* orow = static_cast<char*>(dlogits) + t * ld * Elem<DT>::kBytes;
  bool live = (mask == nullptr) || (mask[t] != 0);
  if (live && (y < 0 || y >= V)) {
    if (tid == 0) atomicOr(flags, kFlagToken);
    live = false;
  }
  // one count array for two different sets: the caller left out n_roll_in; the row is dropped and flagged
  if (live && n_roll == nullptr && in_one_set_only(mask, t)) {
    if (tid == 0) atomicOr(flags, kFlagSets);
    live = false;
  }
  const int64_t gt = row_begin + t;
  double w = 0.0;
  int32_t n = 0, nr = 0;
  if (live && gt < cu[B]) {
    const int i = sample_of_row(cu, B, gt);
    n = n_train[i];
    nr = (n_roll != nullptr) ? n_roll[i] : n;
    w = row_pass_weight(fresh32, i, n, nr, lag[i], hp.xi);
  }
  if (!live || (w == 0.0 && logp == nullptr)) {   // nothing to learn from this row: no read at all
    if (tid == 0) {
      if (logp != nullptr) logp[t] = 0.f;
      row_loss[t] = 0.0;
    }
    row_zero<DT, NT>(orow, V);
    return;
  }
  const char* row = static_cast<const char*>(logits) + t * ld * Elem<DT>::kBytes;
  LaneState st;
  row_lse<DT, NT, U, true, false>(row, V, y, st, &sh_zy);
  double lp, ls, ent;
  block_lse_finish<NT, false>(st, &sh_zy, sh_R, sh_S, nullptr, lp, ls, ent);
  if (tid == 0) {
    const float lp32 = static_cast<float>(lp);
    const float lse32 = static_cast<float>(ls);
    if (logp != nullptr) logp[t] = lp32;
    float c = 0.f;
    double lt = 0.0;
    if (w > 0.0)
      c = coef_and_loss(static_cast<double>(lp32), behav_logp[t], teacher_logp[t], w, n, nr, in_sup_set(mask, t),
                        in_roll_set(mask, t), B, hp, grad_scale, &lt);
    row_loss[t] = lt;
    sh_c = c;
    sh_lseL = lse32 * kLog2e;
    sh_gy = c * expm1f(lp32);
  }
  __syncthreads();
  const float c = sh_c;
  if (c == 0.f) {
    row_zero<DT, NT>(orow, V);
    return;
  }
  row_grad<DT, NT, U, false>(row, orow, V, y, c, sh_lseL, sh_gy);   // non-temporal re-read measured faster
}

// =========================================================================================
// K14R: the same call with the row held in registers between the two passes: 1024 lanes x NV 16-byte vectors
// (NV = 19 holds a 303,872-byte row), one workgroup resident per compute unit.  HBM and the fabric see a single read and a
// single write per row.  A workgroup walks rows blockIdx, blockIdx + gridDim, ...: it requests a whole row, reduces
// it, stores the whole gradient row, then requests the next one, so that a compute unit's reads and writes come in
// turn (the other compute units fill the gaps; a plain copy of this shape is the fastest copy measured on the part).
// Rows longer than 1024 NV vectors do not fit and take fopd_k14_fused.  Without scores
// (fresh32 == nullptr) both kernels take weight 1 for every valid sample: the rows at unit sample weight of
// fopd_loss_fwd_bwd_unit, which needs the logits only once because the scores follow from the log-probs written here.
// =========================================================================================

constexpr int kRegRowThreads = 1024;

// What a workgroup knows about a row before touching its logits.
struct RegRowInfo {
  bool load = false;     // the row's logits are needed (live, and either a weight or a log-prob to report)
  int y = 0;
  double w = 0.0;
  int32_t n = 0, nr = 0;
};

template <int DT, int NV>
__global__ void __launch_bounds__(kRegRowThreads)
fopd_k14_regs(const void* logits, void* dlogits, int64_t T, int V, int64_t ld, const int32_t* token_ids,
              const uint8_t* mask, const float* behav_logp, const float* teacher_logp, const int64_t* cu,
              const int32_t* n_train, const int32_t* n_roll, const int32_t* lag, const float* fresh32, int32_t B,
              int64_t row_begin, fopd_hparams hp, float grad_scale, float* logp, double* row_loss, int32_t* flags) {
  constexpr int NT = kRegRowThreads;
  constexpr int E = Elem<DT>::kPerVec;
  __shared__ float sh_zy;
  __shared__ float sh_R[NT / 64];
  __shared__ float sh_S[NT / 64];
  __shared__ float sh_out[3];                  // c_t, lse_t log2 e, the sampled token's entry
  const int tid = threadIdx.x;
  const int nvec = V / E;                      // <= NT * NV, checked on the host
  const int tail_idx = nvec * E + tid;         // ragged tail: fewer than E elements
  const float kNegInf = -__builtin_inff();

  // the same for every lane of the workgroup
  auto classify = [&](int64_t t) {
    RegRowInfo r;
    if (t >= T) return r;
    r.y = token_ids[t];
    bool live = (mask == nullptr) || (mask[t] != 0);
    if (live && (r.y < 0 || r.y >= V)) {
      if (tid == 0) atomicOr(flags, kFlagToken);
      live = false;
    }
    if (live && n_roll == nullptr && in_one_set_only(mask, t)) {
      if (tid == 0) atomicOr(flags, kFlagSets);
      live = false;
    }
    const int64_t gt = row_begin + t;
    if (live && gt < cu[B]) {
      const int i = sample_of_row(cu, B, gt);
      r.n = n_train[i];
      r.nr = (n_roll != nullptr) ? n_roll[i] : r.n;
      r.w = row_pass_weight(fresh32, i, r.n, r.nr, lag[i], hp.xi);
    }
    r.load = live && !(r.w == 0.0 && logp == nullptr);
    // the same in every lane: kept in scalar registers, the vector registers belong to the row
    r.y = __builtin_amdgcn_readfirstlane(r.y);
    r.n = __builtin_amdgcn_readfirstlane(r.n);
    r.nr = __builtin_amdgcn_readfirstlane(r.nr);
    r.load = __builtin_amdgcn_readfirstlane(r.load ? 1 : 0) != 0;
    const uint64_t wb = __builtin_bit_cast(uint64_t, r.w);
    const uint32_t wlo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(wb));
    const uint32_t whi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(wb >> 32));
    r.w = __builtin_bit_cast(double, (static_cast<uint64_t>(whi) << 32) | wlo);
    return r;
  };
  // Rows are read and written through buffer descriptors (base of the row, extent = its whole 16-byte vectors):
  // a lane's address is the descriptor plus a 32-bit byte offset, lanes past the extent read zeros and their
  // stores are dropped by the hardware, and "no next row" is a descriptor of extent 0.  So the store phase has
  // no branch around a load or a store, and no 64-bit address per lane: the vector registers belong to the row.
  // The offsets are formed where they are used, from a value the compiler must take as new each time (hoisted out
  // of the row loop, the 19 offsets would be spilled around the row).
  const uint32_t row_bytes = static_cast<uint32_t>(nvec) * 16u;
  auto row_of = [&](int64_t t) { return static_cast<const char*>(logits) + t * ld * Elem<DT>::kBytes; };
  auto descriptor = [&](const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(bytes), 0x00020000);
  };
  const uint32_t off0 = static_cast<uint32_t>(tid) * 16u;
  auto lane_off = [&](int u) {
    uint32_t o = off0;
    asm volatile("" : "+v"(o));
    return o + static_cast<uint32_t>(u) * (NT * 16u);
  };
  constexpr int kNonTemporal = 2;              // cache-policy bits of the buffer instructions: nt
  constexpr uint32_t kNegInfPacked = (DT == FOPD_BF16) ? 0xff80ff80u : 0xff800000u;

  // One trip per row, plus one before the first row that only requests it: every trip ends with the loop that
  // stores the current row's gradient (if it has one) and the loop that requests the next row, so the row's
  // registers are written in one place only.
  u32x4 q[NV];
  float tail_x = 0.f;
  RegRowInfo cur;                              // the trip before the first row: nothing to reduce or store
  bool have_row = false;
  int64_t t = static_cast<int64_t>(blockIdx.x) - gridDim.x;
  while (true) {
    const int64_t tn = t + gridDim.x;
    const RegRowInfo nxt = classify(tn);
    const char* nv = row_of(nxt.load ? tn : 0);      // never dereferenced unless nxt.load
    const auto rs_next = descriptor(nv, nxt.load ? row_bytes : 0u);
    char* orow = static_cast<char*>(dlogits) + (have_row ? t : 0) * ld * Elem<DT>::kBytes;
    const int y = cur.y, jy = y / E, ey = y % E;
    float c = 0.f, lseL = 0.f, gy = 0.f;
    if (have_row && !cur.load && tid == 0) {
      if (logp != nullptr) logp[t] = 0.f;
      row_loss[t] = 0.0;
    }
    if (cur.load) {
      LaneState st;
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        // the offset is made to depend on the running sum: the compiler otherwise unpacks all vectors first
        // and accumulates afterwards, which needs the row's registers a second time
        uint32_t o = off0;
        asm volatile("" : "+v"(o) : "v"(st.s));
        const int j = static_cast<int>((o + static_cast<uint32_t>(u) * (NT * 16u)) >> 4);
        u32x4 v = q[u];
        if (j >= nvec) v = u32x4{kNegInfPacked, kNegInfPacked, kNegInfPacked, kNegInfPacked};   // selects
        float x[E];
        unpack<DT>(v, x);
        if (j == jy) {
#pragma unroll
          for (int e = 0; e < E; ++e) {
            if (e == ey) {
              sh_zy = x[e];
              x[e] = kNegInf;
            }
          }
        }
        accumulate<E, false>(x, st);
        __builtin_amdgcn_sched_barrier(0);     // one vector at a time: unpacked early, the row would not fit
      }
      if (tail_idx < V) {
        float x1 = tail_x;
        if (tail_idx == y) {
          sh_zy = x1;
          x1 = kNegInf;
        }
        accumulate<1, false>(&x1, st);
      }
      block_lse_merge<NT, false>(st, sh_R, sh_S, nullptr);
      if (tid == 0) {
        double lp, ls, ent;
        lse_from_partials<false>(&sh_zy, sh_R, sh_S, nullptr, NT / 64, lp, ls, ent);
        const float lp32 = static_cast<float>(lp);
        const float lse32 = static_cast<float>(ls);
        if (logp != nullptr) logp[t] = lp32;
        float c0 = 0.f;
        double lt = 0.0;
        if (cur.w > 0.0)
          c0 = coef_and_loss(static_cast<double>(lp32), behav_logp[t], teacher_logp[t], cur.w, cur.n, cur.nr,
                             in_sup_set(mask, t), in_roll_set(mask, t), B, hp, grad_scale, &lt);
        row_loss[t] = lt;
        sh_out[0] = c0;
        sh_out[1] = lse32 * kLog2e;
        sh_out[2] = c0 * expm1f(lp32);
      }
      __syncthreads();
      c = sh_out[0];
      lseL = sh_out[1];
      gy = sh_out[2];
    }
    const bool grad = (c != 0.f);              // the same in every lane
    const float shiftL = log2f(fabsf(c)) - lseL;
    const uint32_t sign_bits = (c < 0.f) ? ((DT == FOPD_BF16) ? 0x80008000u : 0x80000000u) : 0u;
    const float gy_abs = (c < 0.f) ? -gy : gy;           // the sign is put back with all the others
    if (have_row && !grad) row_zero<DT, NT>(orow, V);
    const auto rs_out = descriptor(orow, grad ? row_bytes : 0u);     // extent 0: every store dropped
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const uint32_t o = lane_off(u);
      if (grad) {
        // |c| 2^t = 2^(t + log2 |c|): the factor goes into the exponent and its sign onto the packed result
        float x[E];
        unpack<DT>(q[u], x);
#pragma unroll
        for (int e = 0; e < E; ++e) x[e] = fast_exp2(fmaf(x[e], kLog2e, shiftL));
        if (static_cast<int>(o >> 4) == jy) {
#pragma unroll
          for (int e = 0; e < E; ++e)
            if (e == ey) x[e] = gy_abs;
        }
        u32x4 packed = pack<DT>(x);
        packed.x ^= sign_bits;
        packed.y ^= sign_bits;
        packed.z ^= sign_bits;
        packed.w ^= sign_bits;
        __builtin_amdgcn_raw_buffer_store_b128(packed, rs_out, o, 0, kNonTemporal);
      }
      __builtin_amdgcn_sched_barrier(0);       // one vector at a time
    }
    // The next row is requested when this row's stores are all out: a compute unit reads a whole row, then writes a
    // whole row.  (Requesting each vector as soon as its register's store has gone, so that the unit's loads and
    // stores overlap, is 6 % slower: 20.6 against 19.4 ms on the benchmark's rows.)
#pragma unroll
    for (int u = 0; u < NV; ++u) q[u] = __builtin_amdgcn_raw_buffer_load_b128(rs_next, lane_off(u), 0, kNonTemporal);
    if (tail_idx < V) {
      if (grad) {
        float g = c * fast_exp2(fmaf(tail_x, kLog2e, -lseL));
        if (tail_idx == y) g = gy;
        store_elem<DT>(orow, tail_idx, g);
      }
      if (nxt.load) tail_x = load_elem<DT>(nv, tail_idx);
    }
    // sh_out is rewritten only after the next row's reduction, which has a barrier of its own
    if (tn >= T) break;
    t = tn;
    cur = nxt;
    have_row = true;
  }
}

// =========================================================================================
// K5 / K6: the same two passes when the rollout drift is the full-vocabulary KL of Eq.
// "kl-diagnostics" as printed, KL(pi^t || pi^r) per row, from a second logits tensor z' (the
// stale checkpoint replayed on the same prefixes).  With d_v = z_v - z'_v and p = softmax(z):
//     lse' - lse = log E_p[e^-d],      KL = E_p[d] + log E_p[e^-d].
// Each tensor has its own running reference (its own maximum), so neither sum can overflow however far
// apart the two rows are: S = sum e_v and W = sum e_v d_v on z's reference, S' = sum e'_v on z''s.
// For close rows (the case the diagnostic is for) KL is far smaller than either log-sum-exp, so the lanes
// also sum U = sum (e'_v 2^(ref' - ref) - e_v) directly: E_p[e^-d - 1] = U / S does not come out as the
// difference of two independently rounded sums.  The finish uses U when every lane's two references stayed
// within 2^+-100 of each other and |U / S| < 1/2, else lse - lse' from the two (reference, sum) pairs.
// =========================================================================================

struct LaneStateKl {
  float r = -1.0e38f, rL = -1.0e38f;      // z:  running maximum; reference = ceil(maximum * log2 e)
  float rs = -1.0e38f, rsL = -1.0e38f;    // z': the same
  float s = 0.f, w = 0.f, u = 0.f;                              // on z's reference
  float ss = 0.f;                                               // on z''s reference
  float c = 1.f;                                                // 2^(rsL - rL), or 0 once the lane is `far`
  bool far = false;                                             // the references were more than 2^100 apart
};

// =========================================================================================
// K4R: the gradient kernel with the row held in registers between its loads and its stores, in the launch shape of
// fopd_k14_regs (1024 lanes x NV 16-byte vectors, one workgroup resident per compute unit, walking rows in steps of
// the grid).  A compute unit then reads a whole row, then writes a whole row, instead of mixing 16-byte reads and
// writes: measured with a plain copy of this shape (hbm_probe, "regs-copy": 5.63 TB/s where 2048 workgroups striding
// over the buffers reach 5.33 in the same process).  Every entry is computed exactly as in fopd_k4_grad: same bits.
// =========================================================================================
// (Requesting a vector of the next row as soon as its register's entry is stored, so that loads and stores of a compute
// unit overlap, is much slower: 28.1 ms against 18.6 ms on the benchmark's rows.)
template <int DT, int NV>
__global__ void __launch_bounds__(1024)
fopd_k4_grad_regs(const void* logits, void* dlogits, int64_t T, int V, int64_t ld, const int32_t* token_ids,
                  const float* lse, const float* logp, const float* coef, int segments, int seg_vecs) {
  // A row longer than 1024 NV vectors is cut into `segments` runs of seg_vecs vectors (<= 1024 NV; the last one may be
  // shorter and also takes the row's ragged end): with lse_t and c_t known, the runs of a row are independent.
  constexpr int E = Elem<DT>::kPerVec;
  constexpr int NT = 1024;
  const int tid = threadIdx.x;
  const int nvec = V / E;
  const int64_t items = T * segments;
  for (int64_t item = blockIdx.x; item < items; item += gridDim.x) {
    const int64_t t = item / segments;
    const int seg = static_cast<int>(item - t * segments);
    const int v0 = seg * seg_vecs;
    const int v1 = min(nvec, v0 + seg_vecs);               // this run: vectors v0 .. v1 - 1
    const bool last = (seg == segments - 1);
    const int idx = nvec * E + tid;                        // ragged end of the row: one entry per lane
    const float c = coef[t];
    const int y = token_ids[t];
    char* orow = static_cast<char*>(dlogits) + t * ld * Elem<DT>::kBytes;
    u32x4* ov = reinterpret_cast<u32x4*>(orow);
    if (c == 0.f || y < 0 || y >= V) {                     // no gradient: zeros, the logits are not read
      const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
      for (int j = v0 + tid; j < v1; j += NT) __builtin_nontemporal_store(zero, ov + j);
      if (last && idx < V) store_elem<DT>(orow, idx, 0.f);
      continue;
    }
    const char* row = static_cast<const char*>(logits) + t * ld * Elem<DT>::kBytes;
    const u32x4* rv = reinterpret_cast<const u32x4*>(row);
    u32x4 q[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int j = v0 + tid + k * NT;
      if (j < v1) q[k] = __builtin_nontemporal_load(rv + j);
    }
    float tail = 0.f;
    if (last && idx < V) tail = load_elem<DT>(row, idx);
    const float lseL = lse[t] * kLog2e;
    const float gy = c * expm1f(logp[t]);                  // the sampled token's entry, accurate as p_y -> 1
    const int jy = y / E, ey = y % E;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int j = v0 + tid + k * NT;
      if (j < v1) {
        float x[E];
        unpack<DT>(q[k], x);
#pragma unroll
        for (int e = 0; e < E; ++e) x[e] = c * fast_exp2(fmaf(x[e], kLog2e, -lseL));
        if (j == jy) {
#pragma unroll
          for (int e = 0; e < E; ++e)
            if (e == ey) x[e] = gy;
        }
        __builtin_nontemporal_store(pack<DT>(x), ov + j);
      }
    }
    if (last && idx < V) {
      float g = c * fast_exp2(fmaf(tail, kLog2e, -lseL));
      if (idx == y) g = gy;
      store_elem<DT>(orow, idx, g);
    }
  }
}

constexpr float kKlRefGap = 100.f;

template <int N>
__device__ __forceinline__ void accumulate_kl(const float* x, const float* xs, LaneStateKl& st) {
  float bm = x[0], bs = xs[0];
#pragma unroll
  for (int i = 1; i < N; ++i) {
    bm = fmaxf(bm, x[i]);
    bs = fmaxf(bs, xs[i]);
  }
  if (bm > st.r || bs > st.rs) {                  // rare after the first few vectors
    // references are whole numbers of log2 units: every rescale below is an exact power of two
    if (bm > st.r) {
      const float nrL = ceilf(bm * kLog2e);
      const float scale = fast_exp2(st.rL - nrL);
      st.s *= scale;
      st.w *= scale;
      st.u *= scale;
      st.r = bm;
      st.rL = nrL;
    }
    if (bs > st.rs) {
      const float nrL = ceilf(bs * kLog2e);
      st.ss *= fast_exp2(st.rsL - nrL);
      st.rs = bs;
      st.rsL = nrL;
    }
    // "seen": the lane has met a finite entry of that tensor.  One tensor seen and the other not (its
    // entries were all -inf so far), or references too far apart for 2^gap: the row's finish will not use U.
    const bool seen = st.r > -1.0e37f, seen_s = st.rs > -1.0e37f;
    const float gap = st.rsL - st.rL;
    if (seen != seen_s || (seen && !(fabsf(gap) <= kKlRefGap))) st.far = true;
    st.c = st.far ? 0.f : fast_exp2(gap);
  }
  // two chains per sum; the first two entries start them (no additions to zero)
  float a0 = 0.f, a1 = 0.f, w0 = 0.f, w1 = 0.f, u0 = 0.f, u1 = 0.f, b0 = 0.f, b1 = 0.f;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const float e = fast_exp2(fmaf(x[i], kLog2e, -st.rL));
    const float es = fast_exp2(fmaf(xs[i], kLog2e, -st.rsL));
    // both -inf (an excluded vocabulary entry) must give d = 0, not NaN
    const float d = floor_minus_inf(x[i]) - floor_minus_inf(xs[i]);
    const float du = fmaf(es, st.c, -e);
    if (i == 0) {
      a0 = e;
      b0 = es;
      w0 = e * d;
      u0 = du;
    } else if (i == 1) {
      a1 = e;
      b1 = es;
      w1 = e * d;
      u1 = du;
    } else if (i & 1) {
      a1 += e;
      b1 += es;
      w1 = fmaf(e, d, w1);
      u1 += du;
    } else {
      a0 += e;
      b0 += es;
      w0 = fmaf(e, d, w0);
      u0 += du;
    }
  }
  st.s += a0 + a1;
  st.ss += b0 + b1;
  st.w += w0 + w1;
  st.u += u0 + u1;
}

template <int DT, int U>
__global__ void __launch_bounds__(kStreamThreads)
fopd_k5_kl(const void* logits, const void* logits_stale, int64_t T, int V, int64_t ld, int64_t ld_stale,
           const int32_t* token_ids, const uint8_t* mask, float* roll_kl, float* logp, float* lse, float* dlse,
           float* logq, int32_t* flags) {
  constexpr int E = Elem<DT>::kPerVec;
  constexpr int NT = kStreamThreads;
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x;
  const int y = token_ids[t];
  bool live = (mask == nullptr) || (mask[t] != 0);
  if (live && (y < 0 || y >= V)) {
    if (tid == 0) atomicOr(flags, kFlagToken);
    live = false;
  }
  if (!live) {
    if (tid == 0) {
      roll_kl[t] = 0.f;
      logp[t] = 0.f;
      lse[t] = 0.f;
      dlse[t] = 0.f;
      if (logq != nullptr) logq[t] = 0.f;
    }
    return;
  }
  __shared__ float sh_zy, sh_zsy;
  __shared__ float sh_R[NT / 64], sh_S[NT / 64], sh_W[NT / 64], sh_U[NT / 64];
  __shared__ float sh_Rs[NT / 64], sh_Ss[NT / 64], sh_F[NT / 64];
  const char* row = static_cast<const char*>(logits) + t * ld * Elem<DT>::kBytes;
  const char* rows = static_cast<const char*>(logits_stale) + t * ld_stale * Elem<DT>::kBytes;
  const u32x4* rv = reinterpret_cast<const u32x4*>(row);
  const u32x4* rsv = reinterpret_cast<const u32x4*>(rows);
  const int nvec = V / E;
  const int jy = y / E, ey = y % E;
  const float kNegInf = -__builtin_inff();
  LaneStateKl st;
  constexpr int U2 = (U > 1) ? U / 2 : 1;      // two tensors: half the vectors of each per trip
  const int ytrip = jy / (U2 * NT);
  int trip = 0;
  int j = tid;
  for (; j + (U2 - 1) * NT < nvec; j += U2 * NT, ++trip) {
    u32x4 q[U2], qs[U2];
#pragma unroll
    for (int u = 0; u < U2; ++u) {
      q[u] = __builtin_nontemporal_load(rv + j + u * NT);
      qs[u] = __builtin_nontemporal_load(rsv + j + u * NT);
    }
    float x[U2 * E], xs[U2 * E];
#pragma unroll
    for (int u = 0; u < U2; ++u) {
      unpack<DT>(q[u], x + u * E);
      unpack<DT>(qs[u], xs + u * E);
    }
    if (trip == ytrip) {
#pragma unroll
      for (int u = 0; u < U2; ++u) {
        if (j + u * NT == jy) {
#pragma unroll
          for (int e = 0; e < E; ++e) {
            if (e == ey) {
              sh_zy = x[u * E + e];
              sh_zsy = xs[u * E + e];
              x[u * E + e] = kNegInf;         // the sampled token is left out of the lane sums
              xs[u * E + e] = kNegInf;
            }
          }
        }
      }
    }
    accumulate_kl<U2 * E>(x, xs, st);
  }
  for (; j < nvec; j += NT) {
    float x[E], xs[E];
    unpack<DT>(__builtin_nontemporal_load(rv + j), x);
    unpack<DT>(__builtin_nontemporal_load(rsv + j), xs);
    if (j == jy) {
#pragma unroll
      for (int e = 0; e < E; ++e) {
        if (e == ey) {
          sh_zy = x[e];
          sh_zsy = xs[e];
          x[e] = kNegInf;
          xs[e] = kNegInf;
        }
      }
    }
    accumulate_kl<E>(x, xs, st);
  }
  {
    const int idx = nvec * E + tid;
    if (idx < V) {
      float x1 = load_elem<DT>(row, idx), xs1 = load_elem<DT>(rows, idx);
      if (idx == y) {
        sh_zy = x1;
        sh_zsy = xs1;
        x1 = kNegInf;
        xs1 = kNegInf;
      }
      accumulate_kl<1>(&x1, &xs1, st);
    }
  }
  const float Rw = wave_max(st.rL), Rsw = wave_max(st.rsL);
  const float scale = fast_exp2(st.rL - Rw);
  const float Sw = wave_sum(st.s * scale), Ww = wave_sum(st.w * scale), Uw = wave_sum(st.u * scale);
  const float Ssw = wave_sum(st.ss * fast_exp2(st.rsL - Rsw));
  const float Fw = wave_max(st.far ? 1.f : 0.f);
  const int lane = tid & 63, wv = tid >> 6;
  if (lane == 0) {
    sh_R[wv] = Rw;
    sh_S[wv] = Sw;
    sh_W[wv] = Ww;
    sh_U[wv] = Uw;
    sh_Rs[wv] = Rsw;
    sh_Ss[wv] = Ssw;
    sh_F[wv] = Fw;
  }
  __syncthreads();
  if (tid == 0) {
    float RR = sh_R[0], RRs = sh_Rs[0], far = sh_F[0];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) {
      RR = fmaxf(RR, sh_R[i]);
      RRs = fmaxf(RRs, sh_Rs[i]);
      far = fmaxf(far, sh_F[i]);
    }
    float SS = 0.f, WW = 0.f, UU = 0.f, SSs = 0.f;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) {
      const float sc = fast_exp2(sh_R[i] - RR);
      SS += sh_S[i] * sc;
      WW += sh_W[i] * sc;
      UU += sh_U[i] * sc;
      SSs += sh_Ss[i] * fast_exp2(sh_Rs[i] - RRs);
    }
    const double L2e = static_cast<double>(kLog2e);
    const double zy = sh_zy, zsy = sh_zsy;
    const double zyL = zy * L2e, zsyL = zsy * L2e;
    // current tensor: log-odds of "not y", lp, lse as in the single-tensor pass
    const double others = static_cast<double>(RR) + log2(static_cast<double>(SS));
    const double a2 = others - zyL;
    const double q = exp2(-fabs(a2));
    const double l1q = log1p(q) * (1.0 / kLn2);
    const double lp = -((a2 > 0.0 ? a2 : 0.0) + l1q) * kLn2;
    const double ls = ((a2 > 0.0 ? others : zyL) + l1q) * kLn2;
    const double p_not = (a2 > 0.0) ? 1.0 / (1.0 + q) : q / (1.0 + q);
    const double p_y = (a2 > 0.0) ? q / (1.0 + q) : 1.0 / (1.0 + q);
    // second tensor: its own log-sum-exp from its own (reference, sum) pair
    const double others_s = static_cast<double>(RRs) + log2(static_cast<double>(SSs));
    const double a2s = others_s - zsyL;
    const double ls_s = ((a2s > 0.0 ? others_s : zsyL) + log1p(exp2(-fabs(a2s))) * (1.0 / kLn2)) * kLn2;
    // E_p[d]: the other tokens through the lane sums, the sampled token directly
    double ed = 0.0;
    if (SS > 0.f) ed = p_not * (static_cast<double>(WW) / static_cast<double>(SS));
    const double dy = fmax(zy, -1.0e30) - fmax(zsy, -1.0e30);
    if (p_y > 0.0) ed += p_y * dy;
    // lse - lse': from E_p[e^-d - 1] summed directly when the rows are close, else from the two pairs
    double dl = ls - ls_s;
    if (far == 0.f && SS > 0.f) {
      const double eu = p_not * (static_cast<double>(UU) / static_cast<double>(SS)) + p_y * expm1(-dy);
      if (fabs(eu) < 0.5) dl = -log1p(eu);
    }
    double kl = ed - dl;
    if (kl < 0.0) kl = 0.0;                       // rounding noise of identical rows
    roll_kl[t] = static_cast<float>(kl);
    logp[t] = static_cast<float>(lp);
    lse[t] = static_cast<float>(ls);
    dlse[t] = static_cast<float>(dl);
    if (logq != nullptr) logq[t] = static_cast<float>(zsy - (ls - dl));   // log softmax(z')[y]
  }
}

// Coefficients of the two-tensor gradient kernel and the row's share of the loss.
//   anchor_is_kl = true   token_kl is the full-vocabulary rollout drift (second tensor = stale logits):
//                         c1 = g pref A_t, c2 = g pref lambda, loss share pref ((lp - lq) + lambda kl)
//   anchor_is_kl = false  token_kl is the distribution-level token loss (second tensor = teacher logits):
//                         c1 = -g pref lambda rho delta, c2 = g pref, loss share pref (kl + lambda k(delta))
__global__ void __launch_bounds__(kStreamThreads)
fopd_coef_loss_kl(const float* logp, const float* token_kl, const float* teacher_logp, const float* behav_logp,
                  const uint8_t* mask, const int64_t* cu, const int32_t* n_train, const int32_t* n_roll,
                  const int32_t* lag, const double* fresh64, const float* fresh32, int64_t T, int32_t B,
                  int64_t row_begin, fopd_hparams hp, float grad_scale, bool anchor_is_kl, float* c1, float* c2,
                  double* partials) {
  __shared__ double sh[kStreamThreads / 64];
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kStreamThreads + threadIdx.x;
  double lt = 0.0;
  if (t < T) {
    float a = 0.f, b = 0.f;
    const bool sup = in_sup_set(mask, t), roll = in_roll_set(mask, t);
    const int64_t gt = row_begin + t;
    if ((sup || roll) && gt < cu[B]) {
      const int i = sample_of_row(cu, B, gt);
      const int32_t n = n_train[i], nr = n_roll[i];
      const double f = (fresh64 != nullptr) ? fresh64[i] : static_cast<double>(fresh32[i]);
      const double w = weight_of(f, n, nr, lag[i], hp.xi);
      if (w > 0.0) {
        const double lp = logp[t], lam = hp.lambda, kl = token_kl[t];
        const double wb = w / static_cast<double>(B);
        const double ps = sup ? wb / static_cast<double>(n) : 0.0;       // share of a U^sup row
        const double pr = roll ? wb / static_cast<double>(nr) : 0.0;     // share of a U^roll row
        const double g = static_cast<double>(grad_scale);
        if (anchor_is_kl) {       // token loss (sampled form) on U^sup, full-vocabulary drift on U^roll
          const double lq = teacher_logp[t];
          a = static_cast<float>(g * ps * (lq - lp));
          b = static_cast<float>(g * pr * lam);
          lt = ps * (lp - lq) + pr * lam * kl;
        } else {                  // distribution-level token loss on U^sup, sampled drift on U^roll
          double rho;
          const double d = lp - static_cast<double>(behav_logp[t]);
          const double k = kl_term(d, &rho);
          a = static_cast<float>(-g * pr * lam * rho * d);
          b = static_cast<float>(g * ps);
          lt = ps * kl + pr * lam * k;
        }
      }
    }
    c1[t] = a;
    c2[t] = b;
  }
  const double tot = block_sum<kStreamThreads>(lt, sh);
  if (threadIdx.x == 0) partials[blockIdx.x] = tot;
}

// K6: dlogits[t,u] = p_u (c1 + c2 (d_u - (lse - lse') - KL_t)) - c1 [u == y], since
// d KL(p||p') / dz_u = p_u (log p_u - log p'_u - KL) and log p_u - log p'_u = d_u - (lse - lse').
template <int DT, int U>
__global__ void __launch_bounds__(kStreamThreads)
fopd_k6_grad_kl(const void* logits, const void* logits_stale, void* dlogits, int64_t T, int V, int64_t ld,
                int64_t ld_stale, const int32_t* token_ids, const float* lse, const float* dlse,
                const float* roll_kl, const float* logp, const float* c1, const float* c2) {
  constexpr int E = Elem<DT>::kPerVec;
  constexpr int NT = kStreamThreads;
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x;
  const float a = c1[t], b = c2[t];
  char* orow = static_cast<char*>(dlogits) + t * ld * Elem<DT>::kBytes;
  if ((a == 0.f && b == 0.f) || token_ids[t] < 0 || token_ids[t] >= V) {   // out of range: flagged earlier
    row_zero<DT, NT>(orow, V);
    return;
  }
  const char* row = static_cast<const char*>(logits) + t * ld * Elem<DT>::kBytes;
  const char* rows = static_cast<const char*>(logits_stale) + t * ld_stale * Elem<DT>::kBytes;
  const u32x4* rv = reinterpret_cast<const u32x4*>(row);
  const u32x4* rsv = reinterpret_cast<const u32x4*>(rows);
  u32x4* ov = reinterpret_cast<u32x4*>(orow);
  const int nvec = V / E;
  const int y = token_ids[t];
  const int jy = y / E, ey = y % E;
  const float lseL = lse[t] * kLog2e;
  const float k0 = a - b * (dlse[t] + roll_kl[t]);     // factor = k0 + c2 d_u
  const float lp = logp[t];
  auto grad_of = [&](float x, float xs) {
    const float d = floor_minus_inf(x) - floor_minus_inf(xs);
    return fast_exp2(fmaf(x, kLog2e, -lseL)) * fmaf(b, d, k0);
  };
  auto grad_y = [&](float x, float xs) {               // c1 (p_y - 1) + c2 p_y (...), accurate as p_y -> 1
    const float d = x - xs;
    return a * expm1f(lp) + b * __expf(lp) * (d - dlse[t] - roll_kl[t]);
  };
  constexpr int U2 = (U > 1) ? U / 2 : 1;
  const int ytrip = jy / (U2 * NT);
  int trip = 0;
  int j = tid;
  for (; j + (U2 - 1) * NT < nvec; j += U2 * NT, ++trip) {
    u32x4 q[U2], qs[U2];
#pragma unroll
    for (int u = 0; u < U2; ++u) {
      q[u] = __builtin_nontemporal_load(rv + j + u * NT);
      qs[u] = __builtin_nontemporal_load(rsv + j + u * NT);
    }
#pragma unroll
    for (int u = 0; u < U2; ++u) {
      float x[E], xs[E], g[E];
      unpack<DT>(q[u], x);
      unpack<DT>(qs[u], xs);
#pragma unroll
      for (int e = 0; e < E; ++e) g[e] = grad_of(x[e], xs[e]);
      if (trip == ytrip && j + u * NT == jy) {
#pragma unroll
        for (int e = 0; e < E; ++e)
          if (e == ey) g[e] = grad_y(x[e], xs[e]);
      }
      __builtin_nontemporal_store(pack<DT>(g), ov + j + u * NT);
    }
  }
  for (; j < nvec; j += NT) {
    float x[E], xs[E], g[E];
    unpack<DT>(__builtin_nontemporal_load(rv + j), x);
    unpack<DT>(__builtin_nontemporal_load(rsv + j), xs);
#pragma unroll
    for (int e = 0; e < E; ++e) g[e] = grad_of(x[e], xs[e]);
    if (j == jy) {
#pragma unroll
      for (int e = 0; e < E; ++e)
        if (e == ey) g[e] = grad_y(x[e], xs[e]);
    }
    __builtin_nontemporal_store(pack<DT>(g), ov + j);
  }
  {
    const int idx = nvec * E + tid;
    if (idx < V) {
      const float x1 = load_elem<DT>(row, idx), xs1 = load_elem<DT>(rows, idx);
      store_elem<DT>(orow, idx, idx == y ? grad_y(x1, xs1) : grad_of(x1, xs1));
    }
  }
}

// =========================================================================================
// Small kernels
// =========================================================================================

__global__ void fopd_clear_flags(int32_t* flags) {
  if (threadIdx.x < 4) flags[threadIdx.x] = 0;
}

// Hands the sticky flag word to a caller-owned int32.
__global__ void fopd_copy_flags(const int32_t* flags, int32_t* out) {
  if (threadIdx.x == 0) out[0] = flags[0];
}

// Exclusive scan of seq_lens into cu[0..B] (int64) with one workgroup; checks signs and the
// total.  need_exact >= 0: the total must equal it; otherwise the total must be >= need_min.
__global__ void __launch_bounds__(kScanThreads)
fopd_scan_seqlens(const int32_t* seq_lens, const int32_t* lag, int32_t B, int64_t need_exact,
                  int64_t need_min, int64_t* cu, int32_t* flags) {
  __shared__ int64_t sh[kScanThreads];
  const int tid = threadIdx.x;
  const int per = (B + kScanThreads - 1) / kScanThreads;
  const int lo = tid * per;
  const int hi = min(lo + per, B);
  int64_t local = 0;
  bool bad_len = false, bad_lag = false;
  for (int i = lo; i < hi; ++i) {
    const int32_t h = seq_lens[i];
    bad_len |= (h < 0);
    local += (h < 0 ? 0 : h);
    if (lag != nullptr) bad_lag |= (lag[i] < 0);
  }
  sh[tid] = local;
  __syncthreads();
  for (int off = 1; off < kScanThreads; off <<= 1) {   // inclusive scan of the per-thread sums
    int64_t add = (tid >= off) ? sh[tid - off] : 0;
    __syncthreads();
    sh[tid] += add;
    __syncthreads();
  }
  int64_t run = sh[tid] - local;                        // exclusive prefix of this thread
  for (int i = lo; i < hi; ++i) {
    cu[i] = run;
    const int32_t h = seq_lens[i];
    run += (h < 0 ? 0 : h);
  }
  if (tid == kScanThreads - 1) {
    const int64_t total = sh[tid];
    cu[B] = total;
    if (need_exact >= 0 ? (total != need_exact) : (total < need_min)) atomicOr(flags, kFlagSegments);
  }
  if (bad_len) atomicOr(flags, kFlagSegments);
  if (bad_lag) atomicOr(flags, kFlagLag);
}

// |U_i^sup| and |U_i^roll| of sample i (one workgroup per sample).
__global__ void __launch_bounds__(kSegThreads)
fopd_count_train(const uint8_t* mask, const int64_t* cu, int64_t T, int32_t* n_train, int32_t* n_roll) {
  __shared__ double sh[kSegThreads / 64];
  const int i = blockIdx.x;
  const int64_t a = cu[i];
  int64_t b = cu[i + 1];
  if (b > T) b = T;
  double cs = 0.0, cr = 0.0;
  for (int64_t t = a + threadIdx.x; t < b; t += kSegThreads) {
    if (in_sup_set(mask, t)) cs += 1.0;
    if (in_roll_set(mask, t)) cr += 1.0;
  }
  const double ts = block_sum<kSegThreads>(cs, sh);
  const double tr = block_sum<kSegThreads>(cr, sh);
  if (threadIdx.x == 0) {
    n_train[i] = static_cast<int32_t>(ts);
    n_roll[i] = static_cast<int32_t>(tr);
  }
}

// One workgroup per sample: D^roll as the token mean over U^roll, D^sup and the token loss as token means
// over U^sup (Eq. "kl-diagnostics", Eq. "sample-aggregated-loss"), then the freshness score; a sample
// with either set empty is invalid and gets zeros (Algorithm 1).
__global__ void __launch_bounds__(kSegThreads)
fopd_segment_stats(const float* logp, const float* behav_logp, const float* roll_kl, const float* ell_term,
                   const float* teacher_logp, const float* teacher_logp_stale, const uint8_t* mask,
                   const int64_t* cu,
                   const int32_t* lag, int64_t T, fopd_hparams hp, int32_t* n_train, int32_t* n_roll, float* D_roll,
                   float* D_sup, float* ell, float* cover, float* cover_roll, float* freshness, double* fresh64,
                   int32_t* n_train_ws, int32_t* n_roll_ws) {
  __shared__ double sh[kSegThreads / 64];
  const int i = blockIdx.x;
  const int64_t a = cu[i];
  int64_t b = cu[i + 1];
  if (b > T) b = T;                      // lengths that overrun T are flagged by the scan
  double sr = 0.0, ss = 0.0, sl = 0.0, cs = 0.0, cr = 0.0;
  for (int64_t t = a + threadIdx.x; t < b; t += kSegThreads) {
    const bool sup = in_sup_set(mask, t), roll = in_roll_set(mask, t);
    if (!sup && !roll) continue;
    const double lp = logp[t];
    if (roll) {
      // rollout drift of the token: full-vocabulary KL if the caller has it, else the sampled estimator
      sr += (roll_kl != nullptr) ? static_cast<double>(roll_kl[t])
                                 : kl_term(lp - static_cast<double>(behav_logp[t]), nullptr);
      cr += 1.0;
    }
    if (sup) {
      // (no teacher log-prob of the sampled token is needed when the token loss is supplied and D^sup is 0)
      const double lq = (teacher_logp != nullptr) ? static_cast<double>(teacher_logp[t]) : 0.0;
      if (teacher_logp_stale != nullptr) ss += kl_term(lq - static_cast<double>(teacher_logp_stale[t]), nullptr);
      // token loss: a distribution-level value if the caller has one, else the sampled-token form
      sl += (ell_term != nullptr) ? static_cast<double>(ell_term[t]) : lp - lq;
      cs += 1.0;
    }
  }
  const double tr = block_sum<kSegThreads>(sr, sh);
  const double ts = block_sum<kSegThreads>(ss, sh);
  const double tl = block_sum<kSegThreads>(sl, sh);
  const double tns = block_sum<kSegThreads>(cs, sh);
  const double tnr = block_sum<kSegThreads>(cr, sh);
  if (threadIdx.x == 0) {
    const int32_t ns = static_cast<int32_t>(tns), nr = static_cast<int32_t>(tnr);
    const int64_t H = cu[i + 1] - a;
    double dr = 0.0, ds = 0.0, el = 0.0, cv = 0.0, cvr = 0.0, f = 0.0;
    if (ns > 0 && nr > 0 && lag[i] >= 0) {       // a negative lag is flagged by the scan; the sample is invalid
      dr = tr / tnr;
      ds = ts / tns;
      el = tl / tns;
      cv = tns / static_cast<double>(H);
      cvr = tnr / static_cast<double>(H);
      // k >= 0 mathematically; clamp the rounding noise of an all-fresh sample
      const double surrogate = static_cast<double>(hp.alpha) * sqrt(dr > 0.0 ? dr : 0.0) +
                               static_cast<double>(hp.beta) * sqrt(ds > 0.0 ? ds : 0.0);
      f = exp(-surrogate) / (static_cast<double>(lag[i]) + 1.0);
    }
    if (n_train != nullptr) n_train[i] = ns;
    if (n_roll != nullptr) n_roll[i] = nr;
    if (n_train_ws != nullptr) n_train_ws[i] = ns;
    if (n_roll_ws != nullptr) n_roll_ws[i] = nr;
    if (D_roll != nullptr) D_roll[i] = static_cast<float>(dr);
    if (D_sup != nullptr) D_sup[i] = static_cast<float>(ds);
    if (ell != nullptr) ell[i] = static_cast<float>(el);
    if (cover != nullptr) cover[i] = static_cast<float>(cv);
    if (cover_roll != nullptr) cover_roll[i] = static_cast<float>(cvr);
    if (freshness != nullptr) freshness[i] = static_cast<float>(f);
    if (fresh64 != nullptr) fresh64[i] = f;
  }
}

// mean_i f_i, mean_i |U_i^roll| / H_i and mean_i |U_i^sup| / H_i over all B samples (one workgroup);
// an invalid sample adds 0 to all three (Algorithm 1).
__global__ void __launch_bounds__(kSegThreads)
fopd_aggregate(const double* fresh64, const int32_t* n_train, const int32_t* n_roll, const int32_t* lag,
               const int64_t* cu, int32_t B, float* agg) {
  __shared__ double sh[kSegThreads / 64];
  double sf = 0.0, sc = 0.0, scr = 0.0;
  for (int i = threadIdx.x; i < B; i += kSegThreads) {
    sf += fresh64[i];
    const int64_t H = cu[i + 1] - cu[i];
    if (n_train[i] > 0 && n_roll[i] > 0 && lag[i] >= 0) {
      sc += static_cast<double>(n_train[i]) / static_cast<double>(H);
      scr += static_cast<double>(n_roll[i]) / static_cast<double>(H);
    }
  }
  const double tf = block_sum<kSegThreads>(sf, sh);
  const double tc = block_sum<kSegThreads>(sc, sh);
  const double tcr = block_sum<kSegThreads>(scr, sh);
  if (threadIdx.x == 0) {
    agg[0] = static_cast<float>(tf / B);
    agg[1] = static_cast<float>(tcr / B);
    agg[2] = static_cast<float>(tc / B);
  }
}

// Per-token gradient coefficient c_t and the block's share of the loss.
__global__ void __launch_bounds__(kStreamThreads)
fopd_coef_loss(const float* logp, const float* behav_logp, const float* teacher_logp,
               const uint8_t* mask, const int64_t* cu, const int32_t* n_train, const int32_t* n_roll,
               const int32_t* lag, const double* fresh64, const float* fresh32, int64_t T, int32_t B,
               int64_t row_begin, fopd_hparams hp, float grad_scale, float* coef, double* partials, int32_t* flags) {
  __shared__ double sh[kStreamThreads / 64];
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kStreamThreads + threadIdx.x;
  double lt = 0.0;
  if (t < T) {
    float c = 0.f;
    const int64_t gt = row_begin + t;
    const bool sup = in_sup_set(mask, t), roll = in_roll_set(mask, t);
    if (n_roll == nullptr && in_one_set_only(mask, t)) {
      atomicOr(flags, kFlagSets);      // one count array for two different sets: the row is dropped
    } else if ((sup || roll) && gt < cu[B]) {
      const int i = sample_of_row(cu, B, gt);
      const int32_t n = n_train[i];
      const int32_t nr = (n_roll != nullptr) ? n_roll[i] : n;
      const double f = (fresh64 != nullptr) ? fresh64[i] : static_cast<double>(fresh32[i]);
      const double w = weight_of(f, n, nr, lag[i], hp.xi);
      if (w > 0.0)
        c = coef_and_loss(logp[t], behav_logp[t], teacher_logp[t], w, n, nr, sup, roll, B, hp, grad_scale, &lt);
    }
    coef[t] = c;
  }
  const double tot = block_sum<kStreamThreads>(lt, sh);
  if (threadIdx.x == 0) partials[blockIdx.x] = tot;
}

// Sums the loss partials in a fixed order; writes the weights and the freshness copy.
__global__ void __launch_bounds__(kSegThreads)
fopd_loss_final(const double* partials, int64_t nparts, const int32_t* n_train, const int32_t* n_roll,
                const int32_t* lag, const double* fresh64, const float* fresh32, int32_t B, float xi, float* loss, float* weights,
                float* freshness) {
  __shared__ double sh[kSegThreads / 64];
  // eight independent partial sums per lane keep eight loads in flight (nparts is T in the
  // two-passes-per-row path); the order of additions is still fixed
  double acc[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
  int64_t i = threadIdx.x;
  for (; i + 7 * kSegThreads < nparts; i += 8 * kSegThreads) {
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] += partials[i + k * kSegThreads];
  }
  for (int k = 0; i < nparts; i += kSegThreads, ++k) acc[k & 7] += partials[i];
  const double s = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
  const double tot = block_sum<kSegThreads>(s, sh);
  if (threadIdx.x == 0) loss[0] = static_cast<float>(tot);
  for (int i = threadIdx.x; i < B; i += kSegThreads) {
    const double f = (fresh64 != nullptr) ? fresh64[i] : static_cast<double>(fresh32[i]);
    if (weights != nullptr)
      weights[i] =
          static_cast<float>(weight_of(f, n_train[i], (n_roll != nullptr) ? n_roll[i] : n_train[i], lag[i], xi));
    if (freshness != nullptr) freshness[i] = static_cast<float>(f);
  }
}

// =========================================================================================
// Teacher stored as k tokens per row (ids and log-probabilities): the distribution-level token loss is the
// reverse KL between the student's and the teacher's distributions coarsened to the events {listed token 1},
// ..., {listed token k}, {any other token} (Eq. "sample-aggregated-loss" with a distribution-level l):
//   l_t = sum_j P_j (log P_j - lq_j) + P_rest (log P_rest - log Q_rest),   Q_rest = max(1 - sum_j e^{lq_j}, floor)
//   d l_t / d z_u = p_u (G_u - l_t),   G_u = log P_b - log Q_b of the event b that holds token u.
// Every token outside the list has the same G, so the gradient row is the ordinary stream c p_u with one
// coefficient per row, corrected at the k listed tokens and at the sampled one.
// =========================================================================================

constexpr int kListThreads = 256;     // four wavefronts, one row each
constexpr int kListRows = kListThreads / 64;
constexpr int kListHeld = 4;          // slots per lane kept in registers between the two loops (k <= 256)

// Per row of U^sup: gathers the listed logits, forms l_t, G_rest - l_t and, per slot, p_j and h_j = p_j (G_j - l_t).
// A slot whose id is outside [0, V) is unused.  Rows outside U^sup (and rows whose sampled token is out of range:
// lse = 0 there) get zeros.  One wavefront per row.  g_rest, and p_list together with h_list, may be NULL (only the
// token loss is wanted).
template <int DT>
__global__ void __launch_bounds__(kListThreads)
fopd_topk_terms(const void* logits, int64_t T, int V, int64_t ld, const int32_t* token_ids, const uint8_t* mask,
                const int32_t* list_ids, const float* list_logp, int k, float rest_floor, const float* lse,
                float* token_loss, float* g_rest, float* p_list, float* h_list) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kListRows + (threadIdx.x >> 6);
  if (t >= T) return;                                      // whole wavefronts; no barrier in this kernel
  const int lane = threadIdx.x & 63;
  const int y = token_ids[t];
  const bool live = in_sup_set(mask, t) && y >= 0 && y < V;
  const char* row = static_cast<const char*>(logits) + t * ld * Elem<DT>::kBytes;
  const int32_t* ids = list_ids + t * k;
  const float* lqs = list_logp + t * k;
  const double ls = lse[t];
  // log P_j - lq_j and P_j of the lane's first kListHeld slots stay in registers for the second loop
  double held_g[kListHeld], held_p[kListHeld];
  double sp = 0.0, sq = 0.0, sl = 0.0;
  if (live) {
    int h = 0;
    for (int j = lane; j < k; j += 64, ++h) {
      const int id = ids[j];
      double pj = 0.0, gj = 0.0;
      if (id >= 0 && id < V) {
        const double lq = lqs[j];
        const double lp = static_cast<double>(load_elem<DT>(row, id)) - ls;
        pj = exp(lp);
        gj = lp - lq;
        sp += pj;
        sq += exp(lq);
        if (pj > 0.0) sl += pj * gj;
      }
      if (h < kListHeld) {
        held_p[h] = pj;
        held_g[h] = gj;
      }
    }
  }
  sp = wave_sum(sp);
  sq = wave_sum(sq);
  sl = wave_sum(sl);
  double ell = 0.0, gr = 0.0;
  if (live) {
    const double p_rest = 1.0 - sp, q_rest = fmax(1.0 - sq, static_cast<double>(rest_floor));
    // The listed probabilities come from fp32 log-probs, so what they leave of 1 is known to about 2e-6 and cannot
    // be told from 0 below 2^-24: the rest's probability is floored there.  An unlisted token then has p_u <= P_rest
    // of that size, and its gradient entry p_u c2 (G_rest - l_t) stays within 1e-5 |c2| of the exact one.
    gr = log(fmax(p_rest, 5.9604644775390625e-8)) - log(q_rest);
    ell = sl + (p_rest > 0.0 ? p_rest * gr : 0.0);
  }
  int h = 0;
  for (int j = lane; p_list != nullptr && j < k; j += 64, ++h) {      // (p_list and h_list come together)
    float pj = 0.f, hj = 0.f;
    if (live) {
      double p, g;
      if (h < kListHeld) {
        p = held_p[h];
        g = held_g[h];
      } else {
        const int id = ids[j];
        p = 0.0;
        g = 0.0;
        if (id >= 0 && id < V) {
          const double lp = static_cast<double>(load_elem<DT>(row, id)) - ls;
          p = exp(lp);
          g = lp - static_cast<double>(lqs[j]);
        }
      }
      pj = static_cast<float>(p);
      hj = (p > 0.0) ? static_cast<float>(p * (g - ell)) : 0.f;
    }
    p_list[t * k + j] = pj;
    h_list[t * k + j] = hj;
  }
  if (lane == 0) {
    token_loss[t] = static_cast<float>(ell);
    if (g_rest != nullptr) g_rest[t] = static_cast<float>(gr - ell);
  }
}

// The stream's coefficient of a row: c1 + c2 (G_rest - l_t).
__global__ void __launch_bounds__(kStreamThreads)
fopd_topk_row_coef(const float* c1, const float* c2, const float* g_rest, int64_t T, float* coef) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kStreamThreads + threadIdx.x;
  if (t < T) coef[t] = static_cast<float>(static_cast<double>(c1[t]) + static_cast<double>(c2[t]) * static_cast<double>(g_rest[t]));
}

// After the gradient stream has written c p_u everywhere (and c expm1(lp) at the sampled token): the k listed
// entries become c1 (p_j - [j is the sampled token]) + c2 h_j, and the sampled token's entry, if it is not listed,
// c1 (p_y - 1) + c2 (G_rest - l_t) p_y.  Rows without a token-loss share (c2 = 0) are already right.  One
// wavefront per row.  out_row != NULL: row t of the inputs is row out_row[t] of dlogits (gradient rows stored densely).
template <int DT>
__global__ void __launch_bounds__(kListThreads)
fopd_topk_fixup(void* dlogits, int64_t T, int V, int64_t ld, const int32_t* token_ids, const int32_t* list_ids, int k,
                const float* logp, const float* c1, const float* c2, const float* g_rest, const float* p_list,
                const float* h_list, const int* out_row) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kListRows + (threadIdx.x >> 6);
  if (t >= T) return;
  const int lane = threadIdx.x & 63;
  const float a = c1[t], b = c2[t];
  const int y = token_ids[t];
  if (b == 0.f || y < 0 || y >= V) return;
  char* orow = static_cast<char*>(dlogits) + (out_row != nullptr ? static_cast<int64_t>(out_row[t]) : t) * ld * Elem<DT>::kBytes;
  const float py_m1 = expm1f(logp[t]);                     // p_y - 1, accurate as p_y -> 1
  bool mine = false;
  for (int j = lane; j < k; j += 64) {
    const int id = list_ids[t * k + j];
    if (id < 0 || id >= V) continue;
    const float pj = p_list[t * k + j], hj = h_list[t * k + j];
    float g;
    if (id == y) {
      mine = true;
      g = fmaf(a, py_m1, b * hj);
    } else {
      g = fmaf(a, pj, b * hj);
    }
    store_elem<DT>(orow, id, g);
  }
  const bool listed = __any(mine ? 1 : 0) != 0;
  if (!listed && lane == 0) store_elem<DT>(orow, y, fmaf(a, py_m1, b * g_rest[t] * (py_m1 + 1.0f)));
}

}  // namespace fopd

#endif  // FOPD_KERNELS_HIP_
