// Output projection fused with the streaming log-sum-exp, for gfx950 (CDNA4).
//
//   fopd_k7_lm_head_lse   z[t, v] = sum_k H[t, k] * W[v, k] on the matrix cores, reduced on the fly to
//                         a running (reference, sum) pair per token; the [T, V] logits never exist
//                         in memory.
//   fopd_k7_finish        the sampled token's logit as one dot product per token, the merge of the
//                         per-strip pairs: lse_t, lp_t = z_{t,y_t} - lse_t.
//
// This is the step in front of the loss pass (pi_theta^t(y | x) of Eq. "kl-diagnostics" is the softmax of
// the projected hidden state), and the only dense contraction near it.
//
// Tiling.  A workgroup of four wavefronts (2 x 2) owns 256 tokens and walks a strip of the vocabulary
// in tiles of 256 rows; each wavefront holds a 128 x 128 block of the tile as 4 x 4 accumulators of
// v_mfma_f32_32x32x16_bf16.  The vocabulary is the M side of the instruction and the tokens the N
// side, because a lane of the 32 x 32 result holds 16 rows of ONE column: the reduction over the
// vocabulary then runs inside a lane and needs a single cross-lane step (the two half-waves).
// Both operands are k-contiguous in memory (hidden [T, d], weight [V, d]), so a lane's 8-element
// fragment is one 16-byte LDS read.  LDS rows are 128 bytes (64 hidden elements); the 16-byte chunk
// index is XOR-ed with the row's low three bits so that fragment reads and tile writes are free of
// bank conflicts.  Two stages of (W tile, H tile) = 128 KB of the CU's 160 KB: global loads of the
// next stage are issued before the MFMAs of the current one and land in registers.

#ifndef FOPD_LM_HEAD_HIP_
#define FOPD_LM_HEAD_HIP_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "fopd_kernels.hip"

namespace fopd {

constexpr int kLmTile = 256;                              // vocabulary rows and token rows of a workgroup tile
constexpr int kLmK = 64;                                  // hidden elements per LDS stage
constexpr int kLmStrips = 8;                              // vocabulary strips = partial pairs per token
constexpr int kLmThreads = 256;
constexpr int kLmOperandBytes = kLmTile * kLmK * 2;       // one operand tile of one stage: 32 KB
constexpr int kLmStageBytes = 2 * kLmOperandBytes;
constexpr int kLmLdsBytes = 2 * kLmStageBytes + 2 * kLmTile * 8;   // + the cross-wave exchange
constexpr float kLmNone = -__builtin_inff();              // "no value yet": the reference of an empty pair

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

// (m, s) <- merge of two running pairs, s in units of exp(. - m).  An empty pair is (-inf, 0); the
// equality tests keep (-inf) - (-inf) out of the arithmetic.
__device__ __forceinline__ void lm_merge(float& m, float& s, float m2, float s2) {
  const float mx = fmaxf(m, m2);
  const float a = (m == mx) ? 1.f : fast_exp2((m - mx) * kLog2e);
  const float b = (m2 == mx) ? 1.f : fast_exp2((m2 - mx) * kLog2e);
  s = s * a + s2 * b;
  m = mx;
}

// 16 bytes at (uniform base) + (per-lane byte offset)
__device__ __forceinline__ u32x4 lm_load(const char* base, uint32_t voff) {
  return *reinterpret_cast<const u32x4*>(base + voff);
}

}  // namespace

// WN = wavefronts along the tokens (2: four 128 x 128 wavefronts; 4: eight 128 x 64 wavefronts, two per SIMD)
template <int WN>
__global__ void __launch_bounds__(128 * WN)
fopd_k7_lm_head_lse(const __bf16* __restrict__ W, int64_t ldw, const __bf16* __restrict__ H, int64_t ldh,
                    int T, int V, int d, float2* __restrict__ partial, int n_token_tiles, int n_vocab_tiles,
                    int64_t t_pad) {
  extern __shared__ __align__(16) unsigned char lm_smem[];
  constexpr int NT = 128 * WN;                         // threads
  constexpr int NJ = 8 / WN;                           // 32-token blocks per wavefront
  constexpr int NL = 2048 / NT;                        // 16-byte chunks per thread, operand and stage
  constexpr int RS = NT / 8;                           // rows between a thread's chunks
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;            // vocabulary half, token part of the tile

  // Workgroups are handed to the eight XCDs in turn (id mod 8).  The 32 that run together on one XCD
  // are 4 token tiles x 8 strips, so that each L2 serves 4 hidden tiles and 8 weight tiles to 32 users.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int strip = (slot >> 2) & 7;
  const int token_tile = ((((slot >> 5) << 3) + xcd) << 2) + (slot & 3);
  if (token_tile >= n_token_tiles) return;             // whole workgroup, before any barrier
  const int vt_begin = static_cast<int>(static_cast<int64_t>(strip) * n_vocab_tiles / kLmStrips);
  const int vt_end = static_cast<int>(static_cast<int64_t>(strip + 1) * n_vocab_tiles / kLmStrips);
  const int t0 = token_tile * kLmTile;
  const int nk = d / kLmK;
  const int n_iter = (vt_end - vt_begin) * nk;

  // global -> LDS copy: thread (row = tid / 8 + RS i, chunk = tid % 8), i < NL, 16 bytes each.
  // Inside the matrices the address is (uniform: tile, i, slab) + (per lane: row-in-32, chunk); a tile
  // that hangs over the end of its matrix takes per-lane row offsets that re-read the last row
  // (those rows are discarded later).  All offsets fit 32 bits (checked on the host).
  const int lrow = tid >> 3, chunk = tid & 7;
  const int st_off = lrow * 128 + ((chunk ^ (lrow & 7)) << 4);
  const char* Wb = reinterpret_cast<const char*>(W);
  const char* Hb = reinterpret_cast<const char*>(H);
  const uint32_t w_lane = static_cast<uint32_t>(lrow * ldw + chunk * 8) * 2u;
  const uint32_t h_lane = static_cast<uint32_t>(lrow * ldh + chunk * 8) * 2u;
  const bool h_ragged = (t0 + kLmTile > T);
  uint32_t h_row[NL];                                  // per-lane row offsets of the hidden tile (bytes)
#pragma unroll
  for (int i = 0; i < NL; ++i)
    h_row[i] = static_cast<uint32_t>(min(t0 + lrow + RS * i, T - 1) * ldh + chunk * 8) * 2u;

  u32x4 ra[NL], rb[NL];
  auto load_stage = [&](int vtile, int ko) {
    const int64_t kb = static_cast<int64_t>(ko) * 2;
    if (vtile * kLmTile + kLmTile <= V) {
      const char* base = Wb + static_cast<int64_t>(vtile) * kLmTile * ldw * 2 + kb;
#pragma unroll
      for (int i = 0; i < NL; ++i) ra[i] = lm_load(base + static_cast<int64_t>(RS * i) * ldw * 2, w_lane);
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int vr = min(vtile * kLmTile + lrow + RS * i, V - 1);
        ra[i] = lm_load(Wb + kb, static_cast<uint32_t>(vr * ldw + chunk * 8) * 2u);
      }
    }
    if (!h_ragged) {
      const char* base = Hb + static_cast<int64_t>(t0) * ldh * 2 + kb;
#pragma unroll
      for (int i = 0; i < NL; ++i) rb[i] = lm_load(base + static_cast<int64_t>(RS * i) * ldh * 2, h_lane);
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) rb[i] = lm_load(Hb + kb, h_row[i]);
    }
  };
  auto store_stage = [&](unsigned char* stage) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      *reinterpret_cast<u32x4*>(stage + st_off + i * RS * 128) = ra[i];
      *reinterpret_cast<u32x4*>(stage + kLmOperandBytes + st_off + i * RS * 128) = rb[i];
    }
  };

  // LDS -> fragment: lane reads row (lane % 32) of a 32-row block, hidden elements
  // 16 ks + 8 (lane / 32) .. + 7, i.e. chunk 2 ks + lane / 32, swizzled by the row's low bits
  const int frag_row = (lane & 31) * 128;
  const int a_off = wm * 128 * 128 + frag_row;
  const int b_off = kLmOperandBytes + wn * NJ * 32 * 128 + frag_row;
  int xk[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) xk[ks] = ((2 * ks + (lane >> 5)) ^ (lane & 7)) << 4;

  f32x16 acc[4][NJ];
  float run_ref[NJ], run_sum[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    run_ref[j] = kLmNone;
    run_sum[j] = 0.f;
  }

  if (n_iter > 0) {
    load_stage(vt_begin, 0);
    store_stage(lm_smem);
  }
  __syncthreads();

  // One finished tile.  Result register r of block (i, j) is vocabulary row
  // 32 i + 8 (r / 4) + 4 (lane / 32) + r % 4 of the wavefront's 128, token 32 j + lane % 32.
  // RAGGED (the last vocabulary tile only): rows at or past V count as "no value".
  auto epilogue = [&](auto ragged_tag, int vlane) {
    constexpr bool RAGGED = decltype(ragged_tag)::value;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      auto value = [&](int i, int r) -> float {
        if (RAGGED && vlane + i * 32 + ((r >> 2) << 3) + (r & 3) >= V) return kLmNone;
        return acc[i][j][r];
      };
      float mx = run_ref[j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, value(i, r));
      // a lane that has seen no value yet (only in a tile that hangs over the vocabulary's end) keeps
      // a finite reference, so that every term below is exp2(-inf) = 0 rather than a NaN
      const float mref = (mx == kLmNone) ? 0.f : mx * kLog2e;
      float s = run_sum[j] * fast_exp2(fmaf(run_ref[j], kLog2e, -mref));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s += fast_exp2(fmaf(value(i, r), kLog2e, -mref));
      }
      run_ref[j] = mx;
      run_sum[j] = s;
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  int it = 0;                                          // stages consumed so far: parity picks the LDS half
  for (int vt = vt_begin; vt < vt_end; ++vt) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int kt = 0; kt < nk; ++kt, ++it) {
      const bool more = (it + 1 < n_iter);
      if (more) {                                      // next stage: (vt, kt + 1) or (vt + 1, 0)
        const bool wrap = (kt + 1 == nk);
        load_stage(wrap ? vt + 1 : vt, wrap ? 0 : (kt + 1) * kLmK);
      }

      const unsigned char* stage = lm_smem + (it & 1) * kLmStageBytes;
      bf16x8 a[2][4], b[2][NJ];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[0][i] = *reinterpret_cast<const bf16x8*>(stage + a_off + i * 4096 + xk[0]);
#pragma unroll
      for (int j = 0; j < NJ; ++j) b[0][j] = *reinterpret_cast<const bf16x8*>(stage + b_off + j * 4096 + xk[0]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        if (ks < 3) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            a[(ks + 1) & 1][i] = *reinterpret_cast<const bf16x8*>(stage + a_off + i * 4096 + xk[(ks + 1) & 3]);
#pragma unroll
          for (int j = 0; j < NJ; ++j)
            b[(ks + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(stage + b_off + j * 4096 + xk[(ks + 1) & 3]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < NJ; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][i], b[ks & 1][j], acc[i][j], 0, 0, 0);
      }

      if (more) store_stage(lm_smem + ((it + 1) & 1) * kLmStageBytes);
      __syncthreads();
    }

    const int vlane = vt * kLmTile + wm * 128 + ((lane >> 5) << 2);
    if (vt * kLmTile + kLmTile > V) epilogue(std::true_type(), vlane);
    else epilogue(std::false_type(), vlane);
  }

  // half-waves, then the two wavefronts that share these tokens, then one pair per token and strip
  float2* ex = reinterpret_cast<float2*>(lm_smem + 2 * kLmStageBytes);
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    float m = run_ref[j], s = run_sum[j];
    const float m2 = __shfl_xor(m, 32), s2 = __shfl_xor(s, 32);
    if (lane < 32) {
      lm_merge(m, s, m2, s2);
      ex[wm * kLmTile + wn * NJ * 32 + j * 32 + lane] = make_float2(m, s);
    }
  }
  __syncthreads();
  if (tid < kLmTile && t0 + tid < T) {
    const float2 e0 = ex[tid], e1 = ex[kLmTile + tid];
    float m = e0.x, s = e0.y;
    lm_merge(m, s, e1.x, e1.y);
    partial[static_cast<int64_t>(strip) * t_pad + t0 + tid] = make_float2(m, s);
  }
}

// One wavefront per token: the sampled token's logit as a dot product of two rows (fp32 products of
// bf16 are exact, the sum is fp32), then the merge of the strip pairs.  lp is clamped at 0 because
// this dot product and the matrix cores sum the same products in different orders.
__global__ void __launch_bounds__(256)
fopd_k7_finish(const __bf16* __restrict__ W, int64_t ldw, const __bf16* __restrict__ H, int64_t ldh,
               const float2* __restrict__ partial, int T, int V, int d, int64_t t_pad,
               const int32_t* __restrict__ token_ids, const uint8_t* __restrict__ mask,
               float* __restrict__ logp, float* __restrict__ lse, int32_t* flags) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const int y = token_ids[t];
  bool live = (mask == nullptr) || (mask[t] != 0);
  if (live && (y < 0 || y >= V)) {
    if (lane == 0) atomicOr(flags, kFlagToken);
    live = false;
  }
  if (!live) {
    if (lane == 0) {
      logp[t] = 0.f;
      lse[t] = 0.f;
    }
    return;
  }
  const __bf16* h = H + static_cast<int64_t>(t) * ldh;
  const __bf16* w = W + static_cast<int64_t>(y) * ldw;
  float dot = 0.f;
  for (int k = lane * 8; k < d; k += 512) {
    const u32x4 hv = *reinterpret_cast<const u32x4*>(h + k);
    const u32x4 wv = *reinterpret_cast<const u32x4*>(w + k);
    float hx[8], wx[8];
    unpack<FOPD_BF16>(hv, hx);
    unpack<FOPD_BF16>(wv, wx);
#pragma unroll
    for (int e = 0; e < 8; ++e) dot = fmaf(hx[e], wx[e], dot);
  }
  dot = wave_sum(dot);
  if (lane == 0) {
    float2 e = partial[t];
    float m = e.x, s = e.y;
#pragma unroll
    for (int k = 1; k < kLmStrips; ++k) {
      e = partial[static_cast<int64_t>(k) * t_pad + t];
      lm_merge(m, s, e.x, e.y);
    }
    const double l = static_cast<double>(m) + log(static_cast<double>(s));
    lse[t] = static_cast<float>(l);
    logp[t] = static_cast<float>(fmin(static_cast<double>(dot) - l, 0.0));
  }
}

}  // namespace fopd

#endif  // FOPD_LM_HEAD_HIP_
