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
// Tiling.  A workgroup of eight wavefronts (2 along the vocabulary x 4 along the tokens, two per SIMD)
// owns 256 tokens and walks a strip of the vocabulary in tiles of 256 rows; each wavefront holds a
// 128 x 64 block of the tile as 4 x 2 accumulators of v_mfma_f32_32x32x16_bf16.  The vocabulary is the
// M side of the instruction and the tokens the N side, because a lane of the 32 x 32 result holds 16
// rows of ONE column: the reduction over the vocabulary then runs inside a lane and needs a single
// cross-lane step (the two half-waves).  Both operands are k-contiguous in memory (hidden [T, d],
// weight [V, d]), so a lane's 8-element fragment is one 16-byte LDS read.
//
// Memory pipeline.  A stage is 32 hidden elements of both tiles (2 x 16 KB); the LDS holds two pairs of
// stages (128 KB of the CU's 160 KB), a pair being 64 hidden elements, i.e. whole 128-byte lines of
// both matrices.  A pair travels global -> vector registers -> LDS in four quarters, one per 16-element slice
// of the pair being multiplied: each slice writes one quarter of the next pair to the LDS and requests the same
// quarter of the pair after it, so every load has a whole pair of matrix work to land and the L1 sees an even
// stream of requests.  (Direct global -> LDS loads, 16 bytes per lane with lane i writing LDS bytes
// [base + 16 i, + 16), were used first: they can only be issued in a burst behind the barrier that frees the
// buffers, which costs 9 % on this loop.)  The slots are those a direct load would fill, so the map below holds.
// Measured on MI355X: this loop is bound by the L1 miss path from the L2, about 17 - 19 bytes per clock and
// compute unit where full MFMA rate on a 256 x 256 tile needs 32 (timing variants and counters: gemm_probe).
// LDS rows are 64 bytes; the LDS serves 16 lanes x 16 bytes per clock (64 banks), so the 16 rows that a
// quarter-wave reads at one logical 16-byte chunk must land on 16 different chunk slots modulo 16:
// the chunk index is XOR-ed with bits 2..3 of the row (rows r .. r + 3 already differ by 4 slots).
// The LDS side of a slot is fixed by the lane number (as a direct load fixes it), so the permutation is applied
// on the global side: lane i fetches the chunk that belongs in slot i.

#ifndef FOPD_LM_HEAD_HIP_
#define FOPD_LM_HEAD_HIP_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "fopd_kernels.hip"

namespace fopd {

constexpr int kLmTile = 256;                              // vocabulary rows and token rows of a workgroup tile
constexpr int kLmK = 32;                                  // hidden elements per LDS stage
constexpr int kLmStages = 4;                              // stages resident in the LDS
constexpr int kLmStripsMax = 32;                          // vocabulary strips (8, 16 or 32) = partial pairs per token
constexpr int kLmThreads = 512;                           // 8 wavefronts: 2 (vocabulary) x 4 (tokens)
constexpr int kLmOperandBytes = kLmTile * kLmK * 2;       // one operand tile of one stage: 16 KB
constexpr int kLmStageBytes = 2 * kLmOperandBytes;
constexpr int kLmLdsBytes = kLmStages * kLmStageBytes + 2 * kLmTile * 8;   // + the cross-wave exchange
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

// 16 bytes per lane from (uniform base) + (per-lane byte offset) straight into the LDS: lane i of the
// wavefront writes lds_base + 16 i (lds_base is the same for all lanes).
__device__ __forceinline__ void lm_load_to_lds(const char* base, uint32_t voff, unsigned char* lds_base) {
  typedef __attribute__((address_space(1))) const void gptr_t;
  typedef __attribute__((address_space(3))) void lptr_t;
  __builtin_amdgcn_global_load_lds((gptr_t*)(base + voff), (lptr_t*)lds_base, 16, 0, 0);
}

}  // namespace

__global__ void __launch_bounds__(kLmThreads)
fopd_k7_lm_head_lse(const __bf16* __restrict__ W, int64_t ldw, const __bf16* __restrict__ H, int64_t ldh,
                    int T, int V, int d, float2* __restrict__ partial, int n_token_tiles, int n_vocab_tiles,
                    int n_strips, int64_t t_pad, const int* __restrict__ row_map, const int* __restrict__ n_live) {
  extern __shared__ __align__(16) unsigned char lm_smem[];
  constexpr int WN = 4;                                // wavefronts along the tokens
  constexpr int NJ = 8 / WN;                           // 32-token blocks per wavefront
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;            // vocabulary half, token quarter of the tile

  // Workgroups are handed to the eight XCDs in turn (id mod 8).  The 32 that run together on one XCD
  // are 4 token tiles x 8 strips, so that each L2 serves 4 hidden tiles and 8 weight tiles to 32 users.
  // With more than 8 strips (shorter work items, a shorter idle tail at the end of the launch) the groups
  // of 8 strips of one set of token tiles follow each other.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int strip_groups = n_strips >> 3;
  const int chunk_id = slot >> 5;
  int strip = ((chunk_id % strip_groups) << 3) + ((slot >> 2) & 7);
  int token_tile = ((((chunk_id / strip_groups) << 3) + xcd) << 2) + (slot & 3);
  if (n_live != nullptr) {
    // Only the rows row_map[0 .. *n_live - 1] of H take part (masked rows left out; the count stays on the device
    // and the launch covers all T): token tile c holds compact rows 256 c .. 256 c + 255, gathered by the loads, and
    // the groups of 4 token tiles x 8 strips are dealt to the XCDs in turn so that they stay evenly loaded.
    T = *n_live;
    if (T <= 0) return;
    n_token_tiles = min(n_token_tiles, (T + kLmTile - 1) / kLmTile);
    const int quads = (n_token_tiles + 3) >> 2;
    const int unit = (chunk_id << 3) + xcd;
    if (unit / quads >= strip_groups) return;
    strip = ((unit / quads) << 3) + ((slot >> 2) & 7);
    token_tile = ((unit % quads) << 2) + (slot & 3);
  }
  if (token_tile >= n_token_tiles) return;             // whole workgroup, before any barrier
  const int vt_begin = static_cast<int>(static_cast<int64_t>(strip) * n_vocab_tiles / n_strips);
  const int vt_end = static_cast<int>(static_cast<int64_t>(strip + 1) * n_vocab_tiles / n_strips);
  const int t0 = token_tile * kLmTile;
  const int nk = d / kLmK;
  const int n_iter = (vt_end - vt_begin) * nk;

  // global -> LDS copy.  An operand tile of a stage is 1024 chunks of 16 bytes = 16 wave instructions;
  // wavefront w issues instructions 2 w and 2 w + 1 of each operand.  Instruction q fills rows
  // 16 q .. 16 q + 15: lane i writes slot (row 16 q + i / 4, physical chunk i % 4) and therefore fetches
  // logical chunk (i % 4) ^ ((i / 16) % 4) of that row.  Rows past the end of a matrix re-read its last
  // row (they are discarded later): the row is clamped, which changes nothing inside the matrix, so
  // the loop has no branch.  All offsets fit 32 bits (checked on the host).
  const int cp_row = wave * 32 + (lane >> 2);          // row of instruction 2 w; instruction 2 w + 1: + 16
  const int cp_chunk = (lane & 3) ^ ((lane >> 4) & 3);
  const int cp_lds = wave * 2048;                      // LDS offset of instruction 2 w inside the operand
  const char* Wb = reinterpret_cast<const char*>(W);
  const char* Hb = reinterpret_cast<const char*>(H) + (row_map != nullptr ? 0 : static_cast<int64_t>(t0) * ldh * 2);
  const uint32_t ldw2 = static_cast<uint32_t>(ldw) * 2u;
  uint32_t h_off[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int r = min(cp_row + 16 * q, T - 1 - t0);
    const uint32_t row = (row_map != nullptr) ? static_cast<uint32_t>(row_map[t0 + r]) : static_cast<uint32_t>(r);
    h_off[q] = row * static_cast<uint32_t>(ldh) * 2u + cp_chunk * 16;
  }

  // The two stages that hold vocabulary tile `vtile`, hidden elements ko .. ko + 63, travel through vector
  // registers in four quarters (ordinary 16-byte loads, then ds_write_b128 to LDS offset 1024 q + 16 lane of
  // instruction q): one quarter = one instruction of one operand, both halves of its 128-byte lines, requested
  // back to back.  Group g = 0, 1: weight rows, instruction 0 / 1; 2, 3: hidden rows.
  u32x4 staged[8];
  auto load_quarter = [&](int vtile, int ko, int g) {
    const int64_t kb = static_cast<int64_t>(ko) * 2;
    const int q = g & 1;
    if (g < 2) {
      const int last = V - 1 - vtile * kLmTile;
      const char* wsrc = Wb + static_cast<int64_t>(vtile) * kLmTile * ldw * 2 + kb;
      const uint32_t w_off = static_cast<uint32_t>(min(cp_row + 16 * q, last)) * ldw2 + cp_chunk * 16;
      staged[2 * g] = *reinterpret_cast<const u32x4*>(wsrc + w_off);
      staged[2 * g + 1] = *reinterpret_cast<const u32x4*>(wsrc + 64 + w_off);
    } else {
      staged[2 * g] = *reinterpret_cast<const u32x4*>(Hb + kb + h_off[q]);
      staged[2 * g + 1] = *reinterpret_cast<const u32x4*>(Hb + kb + 64 + h_off[q]);
    }
  };
  auto write_quarter = [&](int pb, int g) {
    unsigned char* dst = lm_smem + 2 * pb * kLmStageBytes + cp_lds + (g & 1) * 1024 + lane * 16 +
                         (g < 2 ? 0 : kLmOperandBytes);
    *reinterpret_cast<u32x4*>(dst) = staged[2 * g];
    *reinterpret_cast<u32x4*>(dst + kLmStageBytes) = staged[2 * g + 1];
  };

  // LDS -> fragment: lane reads row (lane % 32) of a 32-row block, hidden elements
  // 16 ks + 8 (lane / 32) .. + 7 of the stage, i.e. logical chunk 2 ks + lane / 32
  const int frag_row = (lane & 31) * 64;
  const int a_off = wm * 128 * 64 + frag_row;
  const int b_off = kLmOperandBytes + wn * NJ * 32 * 64 + frag_row;
  int xk[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) xk[ks] = ((2 * ks + (lane >> 5)) ^ ((lane >> 2) & 3)) << 4;

  f32x16 acc[4][NJ];
  float run_ref[NJ], run_sum[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    run_ref[j] = kLmNone;
    run_sum[j] = 0.f;
  }

  // (vt_ld, kt_ld) is the next pair to request; it stops at the last pair, which the tail requests
  // again (never read) instead of branching.
  int vt_ld = vt_begin, kt_ld = 0, s_ld = 0;
  const int n_pairs = n_iter / 2, nkp = nk / 2;
  auto advance_next = [&]() {
    if (s_ld + 1 < n_pairs) {
      ++s_ld;
      if (++kt_ld == nkp) {
        kt_ld = 0;
        ++vt_ld;
      }
    }
  };

  bf16x8 fa[2][4], fb[2][NJ];
  auto read_frags = [&](int buf, const unsigned char* stage, int ks) {
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(stage + a_off + i * 2048 + xk[ks]);
#pragma unroll
    for (int j = 0; j < NJ; ++j) fb[buf][j] = *reinterpret_cast<const bf16x8*>(stage + b_off + j * 2048 + xk[ks]);
  };
  auto multiply = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
  };

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
      const float carried = run_sum[j] * fast_exp2(fmaf(run_ref[j], kLog2e, -mref));
      __builtin_amdgcn_sched_barrier(0);
      float part[4];                                   // four short chains, added as a tree
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        part[i] = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) part[i] += fast_exp2(fmaf(value(i, r), kLog2e, -mref));
      }
      run_ref[j] = mx;
      run_sum[j] = carried + ((part[0] + part[1]) + (part[2] + part[3]));
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Schedule of pair p (buffers 2 (p % 2) and 2 (p % 2) + 1), four 16-element slices.  The registers `staged` hold
  // pair p + 1, requested a whole pair earlier; slice s of pair p
  //   writes quarter s of pair p + 1 to the other pair of buffers (free since the barrier that ended pair p - 1),
  //   requests quarter s of pair p + 2 into the same registers,
  //   reads the fragments of the next slice and multiplies the current one;
  // the one barrier per pair sits in slice 3, after the last write: behind it pair p + 1 is complete and pair p
  // fully read.  Loads and LDS writes are thus spread evenly over the pair (a burst of requests behind each
  // barrier, as direct global -> LDS loads give, costs 9 % on this loop).
  // The order inside a slice is fixed by scheduling group barriers (masks: 0x008 matrix instruction, 0x020 global
  // load, 0x100 LDS read, 0x200 LDS write).  Left to itself the scheduler puts a slice's ten memory instructions ahead
  // of its eight matrix instructions; with one or two of them between consecutive matrix instructions the matrix
  // pipe keeps issuing while they go out.  Measured in one process on the bench shape: 172.6 -> 165.5 ms; one
  // memory instruction per gap 168.4, pairs of writes and of loads per gap 172.6 (no gain).
#define LM_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
  auto interleave = [&]() {
    LM_SGB(0x200, 1); LM_SGB(0x008, 1); LM_SGB(0x200, 1); LM_SGB(0x008, 1);
    LM_SGB(0x020, 1); LM_SGB(0x008, 1); LM_SGB(0x020, 1); LM_SGB(0x008, 1);
    LM_SGB(0x100, 2); LM_SGB(0x008, 1); LM_SGB(0x100, 2); LM_SGB(0x008, 1); LM_SGB(0x100, 2); LM_SGB(0x008, 2);
  };
  if (n_iter > 0) {
#pragma unroll
    for (int g = 0; g < 4; ++g) load_quarter(vt_ld, kt_ld * 64, g);
#pragma unroll
    for (int g = 0; g < 4; ++g) write_quarter(0, g);
    advance_next();
    // in the order the loop keeps (the wait counts at the loop's head assume the less favourable of the two
    // orders that reach it, so a prologue that requests the quarters in another order shortens every wait)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      __builtin_amdgcn_sched_barrier(0);
      load_quarter(vt_ld, kt_ld * 64, g);
    }
    __builtin_amdgcn_sched_barrier(0);
    advance_next();
  }
  __syncthreads();
  if (n_iter > 0) read_frags(0, lm_smem, 0);

  int pit = 0;
  for (int vt = vt_begin; vt < vt_end; ++vt) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int kt = 0; kt < nkp; ++kt, ++pit) {
      const int pb = pit & 1;
      const unsigned char* lo = lm_smem + 2 * pb * kLmStageBytes;
      const unsigned char* hi = lo + kLmStageBytes;
      const unsigned char* next = lm_smem + 2 * (pb ^ 1) * kLmStageBytes;
      const int vt_nx = vt_ld, ko_nx = kt_ld * 64;          // pair p + 2
      write_quarter(pb ^ 1, 0);
      load_quarter(vt_nx, ko_nx, 0);
      read_frags(1, lo, 1);
      multiply(0);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      write_quarter(pb ^ 1, 1);
      load_quarter(vt_nx, ko_nx, 1);
      read_frags(0, hi, 0);
      multiply(1);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      write_quarter(pb ^ 1, 2);
      load_quarter(vt_nx, ko_nx, 2);
      read_frags(1, hi, 1);
      multiply(0);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      write_quarter(pb ^ 1, 3);
      __syncthreads();
      load_quarter(vt_nx, ko_nx, 3);
      advance_next();
      read_frags(0, next, 0);
      multiply(1);
      // behind the barrier: fragment reads in pairs, then the two global loads, between the matrix instructions
      LM_SGB(0x100, 2); LM_SGB(0x008, 1); LM_SGB(0x100, 2); LM_SGB(0x008, 1); LM_SGB(0x100, 2); LM_SGB(0x008, 1);
      LM_SGB(0x020, 1); LM_SGB(0x008, 1); LM_SGB(0x020, 1); LM_SGB(0x008, 4);
      __builtin_amdgcn_sched_barrier(0);
    }

    const int vlane = vt * kLmTile + wm * 128 + ((lane >> 5) << 2);
    if (vt * kLmTile + kLmTile > V) epilogue(std::true_type(), vlane);
    else epilogue(std::false_type(), vlane);
  }

  // half-waves, then the two wavefronts that share these tokens, then one pair per token and strip
  __syncthreads();
  float2* ex = reinterpret_cast<float2*>(lm_smem + kLmStages * kLmStageBytes);
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
// this dot product and the matrix cores sum the same products in different orders.  ex != NULL: only the unmasked
// rows were projected, row t as compact row ex[t] (ex[t] = unmasked rows before row t).
__global__ void __launch_bounds__(256)
fopd_k7_finish(const __bf16* __restrict__ W, int64_t ldw, const __bf16* __restrict__ H, int64_t ldh,
               const float2* __restrict__ partial, int n_strips, int T, int V, int d, int64_t t_pad,
               const int32_t* __restrict__ token_ids, const uint8_t* __restrict__ mask,
               float* __restrict__ logp, float* __restrict__ lse, int32_t* flags, const int* __restrict__ ex) {
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
    const int c = (ex != nullptr) ? ex[t] : t;           // the token's place among the rows that were projected
    float2 e = partial[c];
    float m = e.x, s = e.y;
    for (int k = 1; k < n_strips; ++k) {
      e = partial[static_cast<int64_t>(k) * t_pad + c];
      lm_merge(m, s, e.x, e.y);
    }
    const double l = static_cast<double>(m) + log(static_cast<double>(s));
    lse[t] = static_cast<float>(l);
    logp[t] = static_cast<float>(fmin(static_cast<double>(dot) - l, 0.0));
  }
}

}  // namespace fopd

#endif  // FOPD_LM_HEAD_HIP_
