// Dense bf16 contractions on the matrix cores of gfx950 (CDNA4), and the small kernels around them, for the
// loss pass whose logits are the output projection of the hidden states and are made chunk by chunk:
//
//   fopd_gemm_nt            Out[n, m] (+)= sum_k Bn[n, k] * Am[m, k]     bf16 in, fp32 accumulate, fp32 out
//   fopd_gemm_tn            Out[n, m] (+)= sum_k Bk[k, n] * Ak[k, m]     the same with both operands k-major
//   fopd_transpose_bf16     out[c, r] = in[r, c], zero-padded along r    (brings an operand into k-contiguous form)
//   fopd_k4_grad_wide       gradient rows from fp32 logits to bf16        c_t (softmax(z_t) - onehot)
//
// The three contractions of one chunk of R rows (d hidden size, V vocabulary):
//   logits      Z[R, V]   = H[R, d]  . W[V, d]^T          nt: n = row, m = vocabulary entry, k = hidden element
//   dL/dhidden  dH[R, d]  = dZ[R, V] . (W^T)[d, V]^T      nt: n = row, m = hidden element, k = vocabulary entry
//                                                         (W^T is formed once per call)
//   dL/dweight  dW[V, d] += dZ[R, V]^T . H[R, d]          tn: n = vocabulary entry, m = hidden element, k = row
//
// Tiling and memory pipeline are those of the projection kernel fused with the log-sum-exp
// (fopd_lm_head.hip): a workgroup of eight wavefronts (2 along m x 4 along n) owns a 256 x 256 tile of the
// result; each wavefront holds 128 (m) x 64 (n) of it as 4 x 2 accumulators of v_mfma_f32_32x32x16_bf16;
// stages of 32 k-elements of both operand tiles reach the LDS through vector registers, a quarter of a pair of
// stages per 16-k slice, and are read back as 16-byte fragments through an XOR-swizzled map without bank
// conflicts.  The n-side fragment is the instruction's first operand: the 32 lanes of a half-wave then hold
// consecutive m of one output row, the contiguous side of the output.

#ifndef FOPD_GEMM_HIP_
#define FOPD_GEMM_HIP_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fopd_kernels.hip"
#include "fopd_lm_head.hip"

namespace fopd {

constexpr int kGemmTile = kLmTile;          // 256 x 256 result tile
constexpr int kGemmWavesM = 2, kGemmWavesN = 4;   // eight wavefronts of 128 x 64: the faster of the measured shapes
constexpr int kGemmStaging = 4;                   // operand stages go through registers, a quarter of a pair per slice
constexpr int kGemmThreads = 64 * kGemmWavesM * kGemmWavesN;
// Extent of the result tile along n and bytes of LDS (four stages of both operand tiles) for WN wavefronts along n
// holding TJ 32-row blocks each.
constexpr int gemm_tile_n(int wn, int tj) { return 32 * tj * wn; }
constexpr int gemm_lds_bytes(int wn, int tj) { return kLmStages * (kLmOperandBytes + gemm_tile_n(wn, tj) * 64); }
constexpr int kGemmTileN = gemm_tile_n(kGemmWavesN, 8 / kGemmWavesN);
constexpr int kGemmLdsBytes = gemm_lds_bytes(kGemmWavesN, 8 / kGemmWavesN);

// ACCUMULATE = false: Out = product; true: Out += product (the caller's array holds the running sum).
// K must be a positive multiple of 64; rows past the end of an operand are clamped (re-read) and their
// results discarded.  Byte offsets inside one 256-row operand tile must fit 32 bits (checked on the host).
//
// WM x WN wavefronts share the 256 x 256 tile, each holding (256 / WM) x (256 / WN) of it.  2 x 2 (four
// wavefronts, one per SIMD, 128 x 128 each = 256 accumulator registers) reads a third less from the LDS per
// flop than 2 x 4 (eight wavefronts of 128 x 64): with 2 x 4 the LDS carries 192 KB of fragment reads + 64 KB of
// stage writes per 64 k-elements, as many cycles at 128 bytes per clock as the matrix cores need at full rate.
// Measured, 2 x 4 is the faster shape; the timing variants below show what the loop loses where.
//
// PROBE != 0 are timing variants for the bound analysis (built only into the gemm_probe program; their results
// are wrong on purpose, every access stays inside the same buffers):
//   1  every stage re-reads k = 0..63 of the operand tiles: with direct loads every request is an L2 hit on a hot
//      line (direct loads do not allocate in the L1); with loads through registers every request hits the L1
//   2  no global loads after the prologue: LDS reads + matrix cores only
//   3  global loads as usual, fragments read once: no LDS reads in the loop
//   4  neither: matrix-core issue only
//   5  the first direct-load instruction of the n-side tile left out: 25 % (eight wavefronts) or 12.5 % (four) fewer
//      bytes through the L1, as a wider tile would need per flop
//   6  (register staging only) each line of pair p + 3 is requested once per XCD a pair before its loads, by one of
//      the workgroups that share the tile: lower miss latency, no gain in time
//   7  the wavefront raises its priority while it issues matrix instructions: no gain
//   8  no result stores
//   9  (results correct) non-temporal result stores
//  14  (results correct) the first round of workgroups starts skewed in time (steps of 512 cycles inside an XCD), to
//      spread the bursts of result stores: no gain (steps of 128 and 2048 cycles neither)
//  10  (results correct) no scheduling group barriers: the order inside a slice is the scheduler's (memory instructions
//      first); 11, 13: two other orders (fragment reads first; one memory instruction per gap)
//
// VIA_REGS != 0: the operand stages travel global -> vector registers -> LDS (ordinary loads, then ds_write_b128 to
// the same swizzled slots) instead of global -> LDS directly.  1: the loads of pair p + 2 are issued at the start
// of pair p and written to the LDS at the start of pair p + 1; 2, 3: the same with the loads issued in two / four
// portions over the pair; 4 (shipped): each of the four 16-k slices of a pair writes one quarter of pair p + 1 to
// the LDS and requests the same quarter of pair p + 2, so that every load has a whole pair to land and the L1 sees
// an even stream of requests instead of a burst behind each barrier (measured: 0.45 -> 0.50 of peak).
template <bool ACCUMULATE, int PROBE = 0, int WM = kGemmWavesM, int WN = kGemmWavesN, int TJ = 8 / WN,
          int VIA_REGS = kGemmStaging>
__global__ void __launch_bounds__(64 * WM * WN)
fopd_gemm_nt(const __bf16* __restrict__ Am, int64_t lda, int M, const __bf16* __restrict__ Bn, int64_t ldb, int N,
             int K, float* __restrict__ Out, int64_t ldo, int tiles_m, int tiles_n,
             const int* __restrict__ n_live) {
  extern __shared__ __align__(16) unsigned char gemm_smem[];
  constexpr int WAVES = WM * WN;
  constexpr int TI = 8 / WM;                   // 32-row blocks along m per wavefront
  constexpr int TN = 32 * TJ * WN;             // tile extent along n (TJ 32-row blocks per wavefront): 256, 320 or 384
  constexpr int CPA = 16 / WAVES;              // direct-load instructions per stage and wavefront: m-side tile,
  constexpr int CPB = (TN / 16) / WAVES;       // n-side tile
  constexpr int kABytes = kLmOperandBytes;     // one stage of the m-side tile: 256 rows x 64 bytes
  constexpr int kStage = kABytes + TN * 64;    // one stage of both tiles
  static_assert(WAVES == 4 || WAVES == 8, "four or eight wavefronts");
  static_assert((TN / 16) % WAVES == 0, "the n-side tile must split evenly over the wavefronts");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // Workgroups go to the eight XCDs in turn (id mod 8).  The 32 that an XCD runs together are 4 tiles along n
  // x 8 tiles along m, so that each L2 serves 4 + 8 operand tiles to 32 users.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int m_blocks = (tiles_m + 7) >> 3;
  const int round = slot >> 5;
  int tile_m = ((round % m_blocks) << 3) + ((slot >> 2) & 7);
  int tile_n = ((((round / m_blocks) << 3) + xcd) << 2) + (slot & 3);
  if (n_live != nullptr) {
    // Only the first *n_live rows of Bn count (a device-side count: the launch covers all N): tiles past them are
    // left out, and the groups of 4 x 8 tiles are dealt to the XCDs in turn, the groups along n fastest, so that
    // the XCDs stay evenly loaded whatever the count is.
    const int live = *n_live;
    if (live <= 0) return;
    tiles_n = min(tiles_n, (live + TN - 1) / TN);
    const int quads = (tiles_n + 3) >> 2;
    const int unit = (round << 3) + xcd;
    tile_m = ((unit / quads) << 3) + ((slot >> 2) & 7);
    tile_n = ((unit % quads) << 2) + (slot & 3);
  }
  if (tile_m >= tiles_m || tile_n >= tiles_n) return;      // whole workgroup, before any barrier
  const int m0 = tile_m * kGemmTile, n0 = tile_n * TN;
  if constexpr (PROBE == 14) {
    // the workgroups of the first round start a little apart (those of one XCD 0 .. 31 steps of 512 cycles), so that
    // the result stores of the compute units do not all fall into the same few microseconds
    if (blockIdx.x < 256) {
      const int steps = (blockIdx.x >> 3) & 31;
      for (int i = 0; i < steps; ++i) __builtin_amdgcn_s_sleep(8);
    }
  }

  // global -> LDS copy: see the projection kernel.  An operand tile of a stage is 16 wave instructions of 1 KB;
  // wavefront w issues instructions CPQ w .. CPQ w + CPQ - 1; instruction q fills rows 16 q .. 16 q + 15; lane i
  // writes (row 16 q + i / 4, slot i % 4) and fetches logical 16-byte chunk (i % 4) ^ ((i / 16) % 4) of that row.
  const int cp_chunk = (lane & 3) ^ ((lane >> 4) & 3);
  const char* Ab = reinterpret_cast<const char*>(Am) + static_cast<int64_t>(m0) * lda * 2;
  const char* Bb = reinterpret_cast<const char*>(Bn) + static_cast<int64_t>(n0) * ldb * 2;
  uint32_t a_src[CPA], b_src[CPB];
#pragma unroll
  for (int q = 0; q < CPA; ++q)
    a_src[q] = static_cast<uint32_t>(min((wave * CPA + q) * 16 + (lane >> 2), M - 1 - m0)) * static_cast<uint32_t>(lda) * 2u +
               cp_chunk * 16;
#pragma unroll
  for (int q = 0; q < CPB; ++q)
    b_src[q] = static_cast<uint32_t>(min((wave * CPB + q) * 16 + (lane >> 2), N - 1 - n0)) * static_cast<uint32_t>(ldb) * 2u +
               cp_chunk * 16;
  auto load_pair = [&](int ko, int pb) {
    const int64_t kb = static_cast<int64_t>(ko) * 2;
    unsigned char* dst = gemm_smem + 2 * pb * kStage;
#pragma unroll
    for (int q = 0; q < CPA; ++q) {
      lm_load_to_lds(Ab + kb, a_src[q], dst + (wave * CPA + q) * 1024);
      lm_load_to_lds(Ab + kb + 64, a_src[q], dst + kStage + (wave * CPA + q) * 1024);
    }
#pragma unroll
    for (int q = 0; q < CPB; ++q) {
      if (PROBE == 5 && q == 0) continue;     // a quarter (8 wavefronts) or an eighth (4) of the fill left out
      lm_load_to_lds(Bb + kb, b_src[q], dst + kABytes + (wave * CPB + q) * 1024);
      lm_load_to_lds(Bb + kb + 64, b_src[q], dst + kStage + kABytes + (wave * CPB + q) * 1024);
    }
  };

  // the same stages through vector registers: lane i of instruction q holds what the direct load would have put
  // at LDS offset 1024 q + 16 i
  u32x4 staged[VIA_REGS ? 2 * (CPA + CPB) : 1];
  auto load_regs_a = [&](int ko) {
    const int64_t kb = static_cast<int64_t>(ko) * 2;
#pragma unroll
    for (int q = 0; q < CPA; ++q) {
      staged[2 * q] = *reinterpret_cast<const u32x4*>(Ab + kb + a_src[q]);
      staged[2 * q + 1] = *reinterpret_cast<const u32x4*>(Ab + kb + 64 + a_src[q]);
    }
  };
  auto load_regs_b = [&](int ko) {
    const int64_t kb = static_cast<int64_t>(ko) * 2;
#pragma unroll
    for (int q = 0; q < CPB; ++q) {
      staged[2 * CPA + 2 * q] = *reinterpret_cast<const u32x4*>(Bb + kb + b_src[q]);
      staged[2 * CPA + 2 * q + 1] = *reinterpret_cast<const u32x4*>(Bb + kb + 64 + b_src[q]);
    }
  };
  auto load_regs = [&](int ko) {
    load_regs_a(ko);
    load_regs_b(ko);
  };
  // one quarter of a pair's loads: group g = 0, 1 the first / second half of the m-side instructions, 2, 3 of the n-side
  auto load_regs_quarter = [&](int ko, int g) {
    const int64_t kb = static_cast<int64_t>(ko) * 2;
    if (g < 2) {
#pragma unroll
      for (int q = 0; q < CPA; ++q) {
        if ((q * 2) / CPA != g) continue;
        staged[2 * q] = *reinterpret_cast<const u32x4*>(Ab + kb + a_src[q]);
        staged[2 * q + 1] = *reinterpret_cast<const u32x4*>(Ab + kb + 64 + a_src[q]);
      }
    } else {
#pragma unroll
      for (int q = 0; q < CPB; ++q) {
        if ((q * 2) / CPB != g - 2) continue;
        staged[2 * CPA + 2 * q] = *reinterpret_cast<const u32x4*>(Bb + kb + b_src[q]);
        staged[2 * CPA + 2 * q + 1] = *reinterpret_cast<const u32x4*>(Bb + kb + 64 + b_src[q]);
      }
    }
  };
  auto write_lds = [&](int pb) {
    unsigned char* dst = gemm_smem + 2 * pb * kStage + lane * 16;
#pragma unroll
    for (int q = 0; q < CPA; ++q) {
      *reinterpret_cast<u32x4*>(dst + (wave * CPA + q) * 1024) = staged[2 * q];
      *reinterpret_cast<u32x4*>(dst + kStage + (wave * CPA + q) * 1024) = staged[2 * q + 1];
    }
#pragma unroll
    for (int q = 0; q < CPB; ++q) {
      *reinterpret_cast<u32x4*>(dst + kABytes + (wave * CPB + q) * 1024) = staged[2 * CPA + 2 * q];
      *reinterpret_cast<u32x4*>(dst + kStage + kABytes + (wave * CPB + q) * 1024) = staged[2 * CPA + 2 * q + 1];
    }
  };

  auto write_lds_quarter = [&](int pb, int g) {
    unsigned char* dst = gemm_smem + 2 * pb * kStage + lane * 16;
    if (g < 2) {
#pragma unroll
      for (int q = 0; q < CPA; ++q) {
        if ((q * 2) / CPA != g) continue;
        *reinterpret_cast<u32x4*>(dst + (wave * CPA + q) * 1024) = staged[2 * q];
        *reinterpret_cast<u32x4*>(dst + kStage + (wave * CPA + q) * 1024) = staged[2 * q + 1];
      }
    } else {
#pragma unroll
      for (int q = 0; q < CPB; ++q) {
        if ((q * 2) / CPB != g - 2) continue;
        *reinterpret_cast<u32x4*>(dst + kABytes + (wave * CPB + q) * 1024) = staged[2 * CPA + 2 * q];
        *reinterpret_cast<u32x4*>(dst + kStage + kABytes + (wave * CPB + q) * 1024) = staged[2 * CPA + 2 * q + 1];
      }
    }
  };

  const int frag_row = (lane & 31) * 64;
  const int a_off = wm * TI * 32 * 64 + frag_row;
  const int b_off = kABytes + wn * TJ * 32 * 64 + frag_row;
  int xk[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) xk[ks] = ((2 * ks + (lane >> 5)) ^ ((lane >> 2) & 3)) << 4;

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int n_pairs = K / 64;
  int p_ld = 0;
  auto request_next = [&](int pb) {           // the last pair is requested again at the tail (never read)
    if (PROBE == 2 || PROBE == 4) return;
    load_pair(PROBE == 1 ? 0 : p_ld * 64, pb);
    if (p_ld + 1 < n_pairs) ++p_ld;
  };

  bf16x8 fa[2][TI], fb[2][TJ];
  bool in_loop = false;
  auto read_frags = [&](int buf, const unsigned char* stage, int ks) {
    if ((PROBE == 3 || PROBE == 4) && in_loop) return;
#pragma unroll
    for (int i = 0; i < TI; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(stage + a_off + i * 2048 + xk[ks]);
#pragma unroll
    for (int j = 0; j < TJ; ++j) fb[buf][j] = *reinterpret_cast<const bf16x8*>(stage + b_off + j * 2048 + xk[ks]);
  };
  auto multiply = [&](int buf) {
    if (PROBE == 7) __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
    if (PROBE == 7) __builtin_amdgcn_s_setprio(0);
  };

  // PROBE 10: within a slice, the two LDS writes, the two global loads and the six fragment reads are spread
  // between the eight matrix instructions instead of being left to the scheduler
#define FOPD_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
  // Order of the instructions inside a 16-k slice, fixed by scheduling group barriers (masks: 0x008 matrix
  // instruction, 0x020 global load, 0x100 LDS read, 0x200 LDS write).  Left to itself the scheduler puts a slice's ten
  // memory instructions ahead of its eight matrix instructions; with one or two of them between consecutive matrix
  // instructions the matrix pipe keeps issuing while they go out: 4 - 5 % on the whole loop (gemm_probe).  Slices
  // 0 - 2: the two LDS writes, the two global loads, then the six fragment reads in pairs.  Slice 3 sits behind the
  // barrier: fragment reads in pairs, then the two global loads, each followed by a matrix instruction.
  // (the counts are those of the shipped shape: eight wavefronts, a quarter of a pair per slice)
  constexpr bool kShippedShape = (VIA_REGS == 4 && WAVES == 8 && TJ == 2);
  constexpr int kSched = (!kShippedShape || PROBE == 10) ? 0 : (PROBE == 11) ? 11 : (PROBE == 13) ? 13 : 12;
  auto interleave_tail = [&]() {
    if constexpr (kSched != 0) {
      FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 4);
    }
  };
  auto interleave = [&]() {
    if constexpr (kSched == 11) {           // fragment reads first, then the LDS writes, the loads last
      FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x200, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x200, 1); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 2);
    }
    if constexpr (kSched == 12) {           // shipped
      FOPD_SGB(0x200, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x200, 1); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 2);
    }
    if constexpr (kSched == 13) {           // one memory instruction per gap where there is room
      FOPD_SGB(0x200, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x200, 1); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x100, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1);
    }
  };
  [[maybe_unused]] uint32_t pf_word = 0;
  [[maybe_unused]] const char* pf_base = Ab;
  if constexpr (PROBE == 6) {
    static_assert(PROBE != 6 || (WAVES == 8 && TN == 256 && VIA_REGS == 4), "written for the shipped shape");
    const int u = wave * 12 + min(lane, 11);                 // line 0 .. 95 of this workgroup's share
    if (u < 64) pf_base = Ab + static_cast<int64_t>(min(64 * (slot & 3) + u, M - 1 - m0)) * lda * 2;
    else pf_base = Bb + static_cast<int64_t>(min(32 * ((slot >> 2) & 7) + (u - 64), N - 1 - n0)) * ldb * 2;
  }
  if constexpr (VIA_REGS) {
    // pair 0 into the LDS, pair 1 into registers; then, per pair p: registers (pair p + 1) -> the buffers pair
    // p - 1 has left, loads of pair p + 2 -> registers, multiply pair p, barrier.
    load_regs(0);
    write_lds(0);
    load_regs(n_pairs > 1 ? 64 : 0);
    __syncthreads();
    read_frags(0, gemm_smem, 0);
    for (int p = 0; p < n_pairs; ++p) {
      const int pb = p & 1;
      const unsigned char* lo = gemm_smem + 2 * pb * kStage;
      const unsigned char* hi = lo + kStage;
      const unsigned char* next = gemm_smem + 2 * (pb ^ 1) * kStage;
      // pair p + 2; the last pair again at the tail
      const int k_next = (PROBE == 1) ? 0 : min(p + 2, n_pairs - 1) * 64;
      if (VIA_REGS == 4) {
        // every quarter of pair p + 1 goes to the LDS a whole pair after it was requested, and the request for
        // the same quarter of pair p + 2 follows at once: loads and LDS writes are spread evenly over the pair
        write_lds_quarter(pb ^ 1, 0);
        load_regs_quarter(k_next, 0);
      } else {
        write_lds(pb ^ 1);                                   // pair p + 1 (the compiler waits for its loads)
        if (VIA_REGS == 2) load_regs_a(k_next);
        else if (VIA_REGS == 3) load_regs_quarter(k_next, 0);
        else load_regs(k_next);
      }
      read_frags(1, lo, 1);
      multiply(0);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      if (VIA_REGS == 4) write_lds_quarter(pb ^ 1, 1);
      if (VIA_REGS >= 3) load_regs_quarter(k_next, 1);
      read_frags(0, hi, 0);
      multiply(1);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      if (VIA_REGS == 2) load_regs_b(k_next);
      if (VIA_REGS == 4) write_lds_quarter(pb ^ 1, 2);
      if (VIA_REGS >= 3) load_regs_quarter(k_next, 2);
      read_frags(1, hi, 1);
      multiply(0);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      if (VIA_REGS == 4) write_lds_quarter(pb ^ 1, 3);
      __syncthreads();
      if (VIA_REGS >= 3) load_regs_quarter(k_next, 3);
      if constexpr (PROBE == 6) {
        // pair p + 3 into the L2, a pair before its loads are issued: each of its lines is requested by one of
        // the workgroups that share the operand tile (m-side: 4 workgroups, 64 rows each; n-side: 8, 32 rows each)
        asm volatile("" ::"v"(pf_word));                     // the previous request has returned
        if (lane < 12) pf_word = *reinterpret_cast<const uint32_t*>(pf_base + static_cast<int64_t>(min(p + 3, n_pairs - 1)) * 128);
      }
      read_frags(0, next, 0);
      if constexpr (kSched == 0) __builtin_amdgcn_sched_barrier(0);
      multiply(1);
      interleave_tail();
      if constexpr (kSched != 0) __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    // Same schedule as the projection kernel: two pairs of stages in the LDS; while pair p multiplies, pair p + 1
    // lands; one barrier per pair.  Loads complete in order: after the prologue's two requests (4 CPQ instructions
    // per wavefront each), "at most 4 CPQ outstanding" means pair 0 has landed.
    if (PROBE == 2 || PROBE == 4) {             // the probes without loads still start from loaded stages
      load_pair(0, 0);
      load_pair(0, 1);
    }
    request_next(0);
    request_next(1);
    // "at most one pair's worth of own loads outstanding": 2 (CPA + CPB) instructions per wavefront and pair
    if (PROBE == 5) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (2 * (CPA + CPB) == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (2 * (CPA + CPB) == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (2 * (CPA + CPB) == 18) asm volatile("s_waitcnt vmcnt(18)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(20)" ::: "memory");
    static_assert(2 * (CPA + CPB) == 8 || 2 * (CPA + CPB) == 16 || 2 * (CPA + CPB) == 18 || 2 * (CPA + CPB) == 20,
                  "wait count of the prologue");
    __syncthreads();
    read_frags(0, gemm_smem, 0);
    if (PROBE == 3 || PROBE == 4) read_frags(1, gemm_smem, 1);
    in_loop = true;
    for (int p = 0; p < n_pairs; ++p) {
      const int pb = p & 1;
      const unsigned char* lo = gemm_smem + 2 * pb * kStage;
      const unsigned char* hi = lo + kStage;
      const unsigned char* next = gemm_smem + 2 * (pb ^ 1) * kStage;
      read_frags(1, lo, 1);
      multiply(0);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(0, hi, 0);
      multiply(1);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(1, hi, 1);
      multiply(0);
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      request_next(pb);
      read_frags(0, next, 0);
      __builtin_amdgcn_sched_barrier(0);
      multiply(1);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the tail's unused requests still target the LDS

  }

  if constexpr (PROBE == 8) {                      // no result stores (one conditional store keeps the loop alive)
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
    if (sum == 1.2345e-30f) Out[0] = sum;
    return;
  }
  // The n-side fragment is the matrix instruction's first operand, so register r of block (i, j) is output row
  // n = 32 j + 8 (r / 4) + 4 (lane / 32) + r % 4 of the wavefront's 32 TJ, and the 32 lanes of a half-wave hold
  // consecutive m = 32 i + lane % 32: a store instruction writes two whole 128-byte lines.  (With the m side
  // first, a lane holds four consecutive m and an instruction writes 32 bytes to each of 32 rows: 2 - 3 % slower.)
  const int m = m0 + wm * TI * 32 + (lane & 31);
#pragma unroll
  for (int j = 0; j < TJ; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int n = n0 + wn * TJ * 32 + 32 * j + ((r >> 2) << 3) + ((lane >> 5) << 2) + (r & 3);
      if (n >= N) continue;
      float* orow = Out + static_cast<int64_t>(n) * ldo;
#pragma unroll
      for (int i = 0; i < TI; ++i) {
        if (m + 32 * i < M) {
          if (ACCUMULATE) orow[m + 32 * i] += acc[i][j][r];
          else if (PROBE == 9) __builtin_nontemporal_store(acc[i][j][r], orow + m + 32 * i);
          else orow[m + 32 * i] = acc[i][j][r];
        }
      }
    }
}

// The same contraction with both operands k-major (the contraction index is the row index of both matrices):
//
//   fopd_gemm_tn            Out[n, m] (+)= sum_{k < K} Bk[k, n] * Ak[k, m]
//
// which is the weight gradient as its operands are stored, dW[v, j] += sum_t dZ[t, v] H[t, j], without a transposed
// copy of either.  Tiling, register staging in quarters, barrier placement and the result stores are those of
// fopd_gemm_nt; what differs is the LDS layout and how fragments leave it.  A stage holds 32 k-rows of both
// operand tiles as they are in memory (256 consecutive m or n per row, 512 bytes), row pitch 576 bytes so that
// consecutive rows start 16 banks apart.  A fragment of the matrix instruction (lane = one m, eight consecutive k)
// is two LDS transpose reads (ds_read_b64_tr_b16): within a group of 16 lanes, lane 4 e + q supplies the address of
// four consecutive 16-bit entries and lane i receives entry i % 4 of the lanes 4 e + i / 4, e = 0..3 (measured
// with an in-bounds probe); with lane 4 e + q pointing at row k + e, entries m + 4 q .. 4 q + 3, lane i gets rows
// k .. k + 3 of entry m + i.  The 32 lanes of a pass read 4 rows x 64 bytes: all 64 banks once.
//
// K must be a positive multiple of 64.  Ak has rows_a (1 <= rows_a <= K) readable rows; rows rows_a .. K - 1 are
// taken from row rows_a - 1, so the caller's Bk must hold zeros in every row that is not to count (Bk has K
// readable rows).  M and N need not be multiples of the tile: 16-byte pieces past entry M - 1 / N - 1 of a row are
// clamped (re-read) and their results discarded; M % 8 == 0, lda % 8 == 0, ldb % 8 == 0, and every row of Bk is
// readable up to N rounded up to 8 (ldb is at least that).
constexpr int kTnPitch = 576;                               // bytes per k-row of an operand tile in the LDS
constexpr int kTnOperandBytes = 32 * kTnPitch;              // one operand tile of one stage
constexpr int kTnStageBytes = 2 * kTnOperandBytes;
constexpr int kTnLdsBytes = kLmStages * kTnStageBytes;      // 147,456 of the 163,840 bytes

typedef short tn_i16x4 __attribute__((ext_vector_type(4)));
typedef short tn_i16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ bf16x8 tn_read_fragment(const unsigned char* p) {
  typedef __attribute__((address_space(3))) tn_i16x4* lds_ptr;
  const tn_i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const tn_i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * kTnPitch));
  const tn_i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

template <bool ACCUMULATE, int SCHED = 2>
__global__ void __launch_bounds__(kGemmThreads)
fopd_gemm_tn(const __bf16* __restrict__ Ak, int64_t lda, int M, int rows_a, const __bf16* __restrict__ Bk, int64_t ldb,
             int N, int K, float* __restrict__ Out, int64_t ldo, int tiles_m, int tiles_n,
             const int* __restrict__ k_live) {
  extern __shared__ __align__(16) unsigned char gemm_smem[];
  constexpr int WM = kGemmWavesM, WN = kGemmWavesN, TI = 8 / WM, TJ = 8 / WN;
  if (k_live != nullptr) {
    // only the first *k_live rows of the operands count (a device-side count; the rows after them, up to the next
    // multiple of 64, hold zeros in Bk and finite values in Ak)
    const int live = *k_live;
    if (ACCUMULATE && live <= 0) return;
    K = min(K, max(64, (live + 63) & ~63));
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // tile order: as fopd_gemm_nt (32 workgroups of an XCD = 4 tiles along n x 8 along m)
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int m_blocks = (tiles_m + 7) >> 3;
  const int round = slot >> 5;
  const int tile_m = ((round % m_blocks) << 3) + ((slot >> 2) & 7);
  const int tile_n = ((((round / m_blocks) << 3) + xcd) << 2) + (slot & 3);
  if (tile_m >= tiles_m || tile_n >= tiles_n) return;      // whole workgroup, before any barrier
  const int m0 = tile_m * kGemmTile, n0 = tile_n * kGemmTileN;

  // global -> registers -> LDS.  A pair of stages is 64 k-rows of 512 bytes per operand = 2048 pieces of 16 bytes,
  // four per lane: piece u of stage h is row 32 h + 16 u + tid / 32 of the pair, entries 8 (tid % 32) .. + 7 of
  // the tile; a wave instruction covers two whole rows of the tile.
  const int krow = tid >> 5;
  const int a_piece = min((m0 >> 3) + (tid & 31), (M >> 3) - 1);
  const int b_piece = min((n0 >> 3) + (tid & 31), ((N + 7) >> 3) - 1);
  const char* Ab = reinterpret_cast<const char*>(Ak) + static_cast<int64_t>(a_piece) * 16;
  const char* Bb = reinterpret_cast<const char*>(Bk) + static_cast<int64_t>(b_piece) * 16;
  const int64_t lda2 = lda * 2, ldb2 = ldb * 2;
  const int lds_piece = krow * kTnPitch + (tid & 31) * 16;
  u32x4 staged[8];
  // quarter g of the pair that starts at row k0: g = 0, 1 the m-side operand's stage 0 / 1, g = 2, 3 the n-side's
  auto load_quarter = [&](int k0, int g) {
    const int h = g & 1;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int k = k0 + 32 * h + 16 * u + krow;
      if (g < 2) staged[2 * g + u] = *reinterpret_cast<const u32x4*>(Ab + static_cast<int64_t>(min(k, rows_a - 1)) * lda2);
      else staged[2 * g + u] = *reinterpret_cast<const u32x4*>(Bb + static_cast<int64_t>(k) * ldb2);
    }
  };
  auto write_quarter = [&](int pb, int g) {
    unsigned char* dst = gemm_smem + (2 * pb + (g & 1)) * kTnStageBytes + (g < 2 ? 0 : kTnOperandBytes) + lds_piece;
    *reinterpret_cast<u32x4*>(dst) = staged[2 * g];
    *reinterpret_cast<u32x4*>(dst + 16 * kTnPitch) = staged[2 * g + 1];
  };

  // LDS -> fragment: lane 16 g + 4 e + q points at row 8 (g / 2) + e (+ 4 for the second read), entries
  // 16 (g % 2) + 4 q .. + 3 of a 32-entry block
  const int frag_off = (((lane >> 5) << 3) + ((lane >> 2) & 3)) * kTnPitch + (((lane >> 4) & 1) << 5) + ((lane & 3) << 3);
  const int a_off = frag_off + wm * TI * 64;
  const int b_off = kTnOperandBytes + frag_off + wn * TJ * 64;

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8 fa[2][TI], fb[2][TJ];
  auto read_frags = [&](int buf, const unsigned char* stage, int ks) {
    const unsigned char* base = stage + ks * 16 * kTnPitch;
#pragma unroll
    for (int i = 0; i < TI; ++i) fa[buf][i] = tn_read_fragment(base + a_off + i * 64);
#pragma unroll
    for (int j = 0; j < TJ; ++j) fb[buf][j] = tn_read_fragment(base + b_off + j * 64);
  };
  auto multiply = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
  };

  // the order inside a slice, as in fopd_gemm_nt: the two LDS writes, the two global loads and the twelve transpose
  // reads (four per gap) go between the eight matrix instructions
  // SCHED (timing variants of gemm_probe): 0 the scheduler's own order, 1 reads four per gap behind the writes and
  // loads, 2 two memory instructions in every gap
  auto tn_interleave = [&]() {
    if constexpr (SCHED == 1) {
      FOPD_SGB(0x200, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x200, 1); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x100, 4); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 4); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 4); FOPD_SGB(0x008, 2);
    }
    if constexpr (SCHED == 2) {
      FOPD_SGB(0x200, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x020, 2); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1);
    }
  };

  // pair 0 into the LDS, pair 1 into registers (requested in the order the loop keeps); then per pair p and 16-k
  // slice s: quarter s of pair p + 1 -> LDS, request quarter s of pair p + 2, multiply slice s of pair p
  const int n_pairs = K / 64;
#pragma unroll
  for (int g = 0; g < 4; ++g) load_quarter(0, g);
#pragma unroll
  for (int g = 0; g < 4; ++g) write_quarter(0, g);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    __builtin_amdgcn_sched_barrier(0);
    load_quarter(n_pairs > 1 ? 64 : 0, g);
  }
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  read_frags(0, gemm_smem, 0);
  for (int p = 0; p < n_pairs; ++p) {
    const int pb = p & 1;
    const unsigned char* lo = gemm_smem + 2 * pb * kTnStageBytes;
    const unsigned char* hi = lo + kTnStageBytes;
    const unsigned char* next = gemm_smem + 2 * (pb ^ 1) * kTnStageBytes;
    const int k_next = min(p + 2, n_pairs - 1) * 64;       // pair p + 2; the last pair again at the tail
    write_quarter(pb ^ 1, 0);
    load_quarter(k_next, 0);
    read_frags(1, lo, 1);
    multiply(0);
    tn_interleave();
    __builtin_amdgcn_sched_barrier(0);
    write_quarter(pb ^ 1, 1);
    load_quarter(k_next, 1);
    read_frags(0, hi, 0);
    multiply(1);
    tn_interleave();
    __builtin_amdgcn_sched_barrier(0);
    write_quarter(pb ^ 1, 2);
    load_quarter(k_next, 2);
    read_frags(1, hi, 1);
    multiply(0);
    tn_interleave();
    __builtin_amdgcn_sched_barrier(0);
    write_quarter(pb ^ 1, 3);
    __syncthreads();
    load_quarter(k_next, 3);
    read_frags(0, next, 0);
    if constexpr (SCHED == 0) __builtin_amdgcn_sched_barrier(0);
    multiply(1);
    // behind the barrier: the transpose reads, then the two global loads, between the matrix instructions
    if constexpr (SCHED == 1) {
      FOPD_SGB(0x100, 4); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 4); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 4); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 1); FOPD_SGB(0x020, 1); FOPD_SGB(0x008, 4);
    }
    if constexpr (SCHED == 2) {
      FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1); FOPD_SGB(0x100, 2); FOPD_SGB(0x008, 1);
      FOPD_SGB(0x020, 2); FOPD_SGB(0x008, 2);
    }
    if constexpr (SCHED != 0) __builtin_amdgcn_sched_barrier(0);
  }

  // result stores: as fopd_gemm_nt (register r of block (i, j): n = 32 j + 8 (r / 4) + 4 (lane / 32) + r % 4,
  // m = 32 i + lane % 32)
  const int m = m0 + wm * TI * 32 + (lane & 31);
#pragma unroll
  for (int j = 0; j < TJ; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int n = n0 + wn * TJ * 32 + 32 * j + ((r >> 2) << 3) + ((lane >> 5) << 2) + (r & 3);
      if (n >= N) continue;
      float* orow = Out + static_cast<int64_t>(n) * ldo;
#pragma unroll
      for (int i = 0; i < TI; ++i) {
        if (m + 32 * i < M) {
          // (every entry of Out belongs to one lane of one workgroup, so the hardware add below, which does not
          // wait for the old value to come back, gives the same sums as load - add - store, in the same order)
          if (ACCUMULATE) unsafeAtomicAdd(orow + m + 32 * i, acc[i][j][r]);
          else orow[m + 32 * i] = acc[i][j][r];
        }
      }
    }
}

// out[c, r] = in[r, c] for r < rows, c < cols; out[c, r] = 0 for rows <= r < rows_pad.  64 x 64 tiles through
// the LDS; grid (ceil(rows_pad / 64), ceil(cols / 64)), 256 lanes.
__global__ void __launch_bounds__(256)
fopd_transpose_bf16(const uint16_t* __restrict__ in, int64_t ld_in, int rows, int cols, uint16_t* __restrict__ out,
                    int64_t ld_out, int rows_pad) {
  __shared__ uint16_t tile[64][66];
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int rr = ty; rr < 64; rr += 4) {
    const int r = r0 + rr, c = c0 + tx;
    tile[rr][tx] = (r < rows && c < cols) ? in[static_cast<int64_t>(r) * ld_in + c] : static_cast<uint16_t>(0);
  }
  __syncthreads();
  for (int cc = ty; cc < 64; cc += 4) {
    const int c = c0 + cc, r = r0 + tx;
    if (c < cols && r < rows_pad) out[static_cast<int64_t>(c) * ld_out + r] = tile[tx][cc];
  }
}

// Gradient rows of one chunk from fp32 logits (ldz floats per row) to bf16 (ldg entries per row):
//   g[t, v] = c_t (exp(z[t, v] - lse_t) - [v == y_t]),  columns V .. ldg - 1 written as zeros
// (they are the zero padding of the contraction that follows).  One workgroup per row; rows with c_t == 0 or
// an out-of-range token id are zero-filled without reading the logits.  With grad_ex (grad_ex[t] = rows that have
// a gradient row before row t, t = 0 .. rows) the rows that have one (grad_ex[t + 1] > grad_ex[t]) are written
// densely, row t to row grad_ex[t] of G, and the others not at all.
__global__ void __launch_bounds__(kGradThreads)
fopd_k4_grad_wide(const float* __restrict__ Z, int64_t ldz, uint16_t* __restrict__ G, int64_t ldg, int V,
                  const int32_t* __restrict__ token_ids, const float* __restrict__ lse,
                  const float* __restrict__ logp, const float* __restrict__ coef,
                  const int* __restrict__ grad_ex) {
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x;
  const float c = coef[t];
  const int y = token_ids[t];
  int64_t out = t;
  if (grad_ex != nullptr) {
    out = grad_ex[t];
    if (grad_ex[t + 1] == out) return;
  }
  uint16_t* orow = G + out * ldg;
  u32x4* ov = reinterpret_cast<u32x4*>(orow);
  const int nvec_out = static_cast<int>(ldg / 8);
  if (c == 0.f || y < 0 || y >= V) {
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
    for (int j = tid; j < nvec_out; j += kGradThreads) __builtin_nontemporal_store(zero, ov + j);
    return;
  }
  const float lseL = lse[t] * kLog2e;
  const float gy = c * expm1f(logp[t]);
  const float* zrow = Z + t * ldz;
  const u32x4* zv = reinterpret_cast<const u32x4*>(zrow);
  const int nfull = V / 8;                       // output vectors made of eight existing logits
  for (int j = tid; j < nfull; j += kGradThreads) {
    const u32x4 q0 = __builtin_nontemporal_load(zv + 2 * j);
    const u32x4 q1 = __builtin_nontemporal_load(zv + 2 * j + 1);
    float x[8];
    unpack<FOPD_F32>(q0, x);
    unpack<FOPD_F32>(q1, x + 4);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = c * fast_exp2(fmaf(x[e], kLog2e, -lseL));
    if (j == (y >> 3)) {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e == (y & 7)) x[e] = gy;
    }
    __builtin_nontemporal_store(pack<FOPD_BF16>(x), ov + j);
  }
  for (int v = nfull * 8 + tid; v < static_cast<int>(ldg); v += kGradThreads) {    // ragged tail, then the padding
    float g = 0.f;
    if (v < V) {
      g = c * fast_exp2(fmaf(zrow[v], kLog2e, -lseL));
      if (v == y) g = gy;
    }
    store_elem<FOPD_BF16>(orow, v, g);
  }
}

// Zeroes the first `cols` entries of every row (one workgroup per row) of an fp32 matrix.
__global__ void __launch_bounds__(256) fopd_fill_zero_f32(float* out, int64_t ld, int cols) {
  float* row = out + static_cast<int64_t>(blockIdx.x) * ld;
  for (int c = threadIdx.x; c < cols; c += 256) row[c] = 0.f;
}

// ---- rows that take part moved to the front of a chunk, so that the contractions skip the others ----
// Masked rows (observations, prompts) have no log-prob and no gradient row: the chunk's per-row inputs and hidden
// states are gathered into dense arrays of the live rows (mask != 0), every kernel of the chunk runs on those, and
// the per-row outputs are scattered back (zeros at masked rows).  With scores supplied the live rows of the whole
// call are numbered once and the chunks are runs of that numbering, so that every chunk but the last is full; with
// the scores formed inside, the chunks are whole samples and each is numbered by itself.  Once the coefficients are known the same is done
// again for the gradient side: only the rows with c_t != 0 (not those of samples the freshness weight gates out)
// get a gradient row, written densely, and the two gradient contractions run on those.  The counts stay on the
// device: the launches cover the whole chunk, the contraction kernels read the count and leave out the rest.

constexpr int kLiveScanThreads = 1024;

// keep[i] = 1 if sample i has a positive weight under the scores given (float64 ones if fresh64 != NULL, else the
// float32 ones), else 0.
__global__ void __launch_bounds__(256)
fopd_sample_keep(const double* __restrict__ fresh64, const float* __restrict__ fresh32,
                 const int32_t* __restrict__ n_train, const int32_t* __restrict__ n_roll,
                 const int32_t* __restrict__ lag, int B, float xi, int* __restrict__ keep) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= B) return;
  const int32_t n = n_train[i];
  const double f = (fresh64 != nullptr) ? fresh64[i] : static_cast<double>(fresh32[i]);
  keep[i] = weight_of(f, n, (n_roll != nullptr) ? n_roll[i] : n, lag[i], xi) > 0.0 ? 1 : 0;
}

// One workgroup.  A row is live if coef != NULL ? (coef[j] != 0 or, with coef2, coef2[j] != 0) : (mask == NULL ||
// mask[j] != 0) and, with keep, keep[sample of row row_begin + j] != 0; mask / coef / coef2 point at the chunk's
// first row.  ex[j] = live rows before chunk row j, j = 0 .. R; row_map[c] = chunk row of compact row c
// (row_map may be NULL); n_live[0] = ex[R]; cu_c[i] = ex[clamp(cu[i] - row_begin, 0, R)], i = 0 .. B: the samples'
// offsets among the chunk's live rows (B < 0: none wanted).
__global__ void __launch_bounds__(kLiveScanThreads)
fopd_live_scan(const uint8_t* __restrict__ mask, const float* __restrict__ coef, const float* __restrict__ coef2, int R,
               const int64_t* __restrict__ cu,
               int B, int64_t row_begin, int* __restrict__ ex, int* __restrict__ row_map, int* __restrict__ n_live,
               int64_t* __restrict__ cu_c, const int* __restrict__ keep) {
  __shared__ int wave_total[kLiveScanThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  auto is_live = [&](int j) {
    if (coef != nullptr) return coef[j] != 0.f || (coef2 != nullptr && coef2[j] != 0.f);
    if (mask != nullptr && mask[j] == 0) return false;
    return keep == nullptr || keep[sample_of_row(cu, B, row_begin + j)] != 0;
  };
  // 1024 rows at a time, row base + tid to lane tid (reads and writes of consecutive lanes are consecutive): a
  // wavefront's ballot gives each lane its place among the wavefront's live rows, the sixteen totals give the rest
  int run = 0;
  for (int64_t base = 0; base < R; base += kLiveScanThreads) {
    const int64_t j = base + tid;
    const bool live = j < R && is_live(static_cast<int>(j));
    const unsigned long long votes = __ballot(live);
    const int before_lane = __popcll(votes & ((1ull << lane) - 1ull));
    if (lane == 0) wave_total[wave] = __popcll(votes);
    __syncthreads();
    int before_wave = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kLiveScanThreads / 64; ++w) {
      const int n = wave_total[w];
      before_wave += (w < wave) ? n : 0;
      all += n;
    }
    if (j < R) {
      const int at = run + before_wave + before_lane;
      ex[j] = at;
      if (live && row_map != nullptr) row_map[at] = static_cast<int>(j);
    }
    run += all;
    __syncthreads();                                         // before the totals are overwritten
  }
  if (tid == 0) {
    ex[R] = run;
    n_live[0] = run;
  }
  __syncthreads();                                           // ex[] of the other lanes is visible from here on
  for (int i = tid; i <= B; i += kLiveScanThreads) {
    int64_t j = cu[i] - row_begin;
    j = j < 0 ? 0 : (j > R ? R : j);
    cu_c[i] = ex[j];
  }
}

// Dense row c = blockIdx.x of a chunk (c < gridDim.x) is live row map_off + c of the scan: row row_base +
// row_map[map_off + c] of the caller's arrays if map_off + c < n_live[0], else a masked row of zeros.  Gathers the
// per-row inputs, the listed teacher and the hidden row; the arrays are the caller's (first row), not the chunk's;
// teacher_logp, teacher_stale and the list may be NULL.  n_chunk[0] = the chunk's live rows (what the contraction
// kernels read).  d % 8 == 0.
__global__ void __launch_bounds__(256)
fopd_live_gather(const int* __restrict__ row_map, const int* __restrict__ n_live, int64_t map_off, int64_t row_base,
                 int* __restrict__ n_chunk, const int32_t* __restrict__ token_ids, const uint8_t* __restrict__ mask,
                 const float* __restrict__ behav_logp, const float* __restrict__ teacher_logp,
                 const float* __restrict__ teacher_stale, const int32_t* __restrict__ list_ids,
                 const float* __restrict__ list_logp, int k, const uint16_t* __restrict__ hidden, int64_t ldh, int d,
                 int32_t* __restrict__ token_ids_c, uint8_t* __restrict__ mask_c, float* __restrict__ behav_c,
                 float* __restrict__ teacher_c, float* __restrict__ stale_c, int32_t* __restrict__ list_ids_c,
                 float* __restrict__ list_logp_c, uint16_t* __restrict__ hidden_c) {
  const int64_t c = blockIdx.x;
  const int tid = threadIdx.x;
  const int64_t total = n_live[0];
  const bool live = map_off + c < total;
  const int64_t j = live ? row_base + row_map[map_off + c] : 0;
  if (tid == 0) {
    if (c == 0) {
      const int64_t here = total - map_off;
      n_chunk[0] = static_cast<int>(here < 0 ? 0 : (here > gridDim.x ? gridDim.x : here));
    }
    token_ids_c[c] = live ? token_ids[j] : 0;
    mask_c[c] = live ? (mask != nullptr ? mask[j] : static_cast<uint8_t>(1)) : static_cast<uint8_t>(0);
    behav_c[c] = live ? behav_logp[j] : 0.f;
    if (teacher_logp != nullptr) teacher_c[c] = live ? teacher_logp[j] : 0.f;
    if (teacher_stale != nullptr) stale_c[c] = live ? teacher_stale[j] : 0.f;
  }
  if (list_ids != nullptr) {
    for (int q = tid; q < k; q += 256) {
      list_ids_c[c * k + q] = live ? list_ids[j * k + q] : -1;
      list_logp_c[c * k + q] = live ? list_logp[j * k + q] : 0.f;
    }
  }
  const u32x4* src = reinterpret_cast<const u32x4*>(hidden + j * ldh);
  u32x4* dst = reinterpret_cast<u32x4*>(hidden_c + c * d);
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  for (int v = tid; v < d / 8; v += 256) dst[v] = live ? src[v] : zero;
}

// The hidden rows of the compact rows that have a gradient (grad_ex[c + 1] > grad_ex[c]), densely: row c of hidden_c
// to row grad_ex[c] of hidden_g (d entries per row, d % 8 == 0).  Grid: one workgroup per compact row.
__global__ void __launch_bounds__(256)
fopd_grad_gather(const int* __restrict__ grad_ex, const uint16_t* __restrict__ hidden_c, int64_t ldh, int d,
                 uint16_t* __restrict__ hidden_g) {
  const int64_t c = blockIdx.x;
  const int g = grad_ex[c];
  if (grad_ex[c + 1] == g) return;
  const u32x4* src = reinterpret_cast<const u32x4*>(hidden_c + c * ldh);
  u32x4* dst = reinterpret_cast<u32x4*>(hidden_g + static_cast<int64_t>(g) * d);
  for (int v = threadIdx.x; v < d / 8; v += 256) dst[v] = src[v];
}

// Zeros behind the rows that have a gradient, up to the next multiple of 64 (at least 64 rows in all): the
// contraction over rows reads that far.  Row n_grad[0] + blockIdx.x of G (ldg entries, ldg % 8 == 0) and of hidden_g
// (d entries); grid: 64 workgroups.
__global__ void __launch_bounds__(256)
fopd_grad_tail_zero(const int* __restrict__ n_grad, uint16_t* __restrict__ G, int64_t ldg,
                    uint16_t* __restrict__ hidden_g, int d) {
  const int n = n_grad[0];
  const int64_t row = static_cast<int64_t>(n) + blockIdx.x;
  if (row >= max(64, (n + 63) & ~63)) return;
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  u32x4* g = reinterpret_cast<u32x4*>(G + row * ldg);
  for (int v = threadIdx.x; v < static_cast<int>(ldg / 8); v += 256) g[v] = zero;
  u32x4* h = reinterpret_cast<u32x4*>(hidden_g + row * d);
  for (int v = threadIdx.x; v < d / 8; v += 256) h[v] = zero;
}

// Dense row c = blockIdx.x of a chunk hands its outputs to the caller's row row_base + row_map[map_off + c] (nothing
// if map_off + c >= n_live[0]): log-prob and log-sum-exp (logp, lse: NULL together), token loss, and as dL/dhidden row the dense gradient row
// grad_ex[c] of dhidden_g if the row has one (grad_ex[c + 1] > grad_ex[c]), zeros if not.  token_loss / token_loss_c
// and dhidden / dhidden_g / grad_ex may be NULL.
__global__ void __launch_bounds__(256)
fopd_live_scatter(const int* __restrict__ row_map, const int* __restrict__ n_live, int64_t map_off, int64_t row_base,
                  const float* __restrict__ logp_c, const float* __restrict__ lse_c,
                  const float* __restrict__ token_loss_c, const int* __restrict__ grad_ex,
                  const float* __restrict__ dhidden_g, int d, float* __restrict__ logp, float* __restrict__ lse,
                  float* __restrict__ token_loss, float* __restrict__ dhidden, int64_t lddh) {
  const int64_t c = blockIdx.x;
  const int tid = threadIdx.x;
  if (map_off + c >= n_live[0]) return;
  const int64_t t = row_base + row_map[map_off + c];
  if (tid == 0) {
    if (logp != nullptr) {
      logp[t] = logp_c[c];
      lse[t] = lse_c[c];
    }
    if (token_loss != nullptr) token_loss[t] = token_loss_c[c];
  }
  if (dhidden != nullptr) {
    const int g = grad_ex[c];
    const bool has = grad_ex[c + 1] > g;
    const float* src = dhidden_g + static_cast<int64_t>(g) * d;
    float* dst = dhidden + t * lddh;
    for (int v = tid; v < d; v += 256) dst[v] = has ? src[v] : 0.f;
  }
}

// Zeros in the outputs of the rows 0 .. gridDim.x - 1 that take no part: masked ones (mask != NULL and mask[r] == 0)
// and, with keep, those of samples with keep[i] == 0 (cu: the samples' offsets).  Log-prob and log-sum-exp (NULL
// together), token loss (may be NULL), dL/dhidden row (may be NULL).
__global__ void __launch_bounds__(256)
fopd_masked_rows_zero(const uint8_t* __restrict__ mask, const int64_t* __restrict__ cu, int B,
                      const int* __restrict__ keep, float* __restrict__ logp, float* __restrict__ lse,
                      float* __restrict__ token_loss, float* __restrict__ dhidden, int64_t lddh, int d) {
  const int64_t r = blockIdx.x;
  const bool masked = (mask != nullptr && mask[r] == 0);
  if (!masked && (keep == nullptr || keep[sample_of_row(cu, B, r)] != 0)) return;
  if (threadIdx.x == 0) {
    if (logp != nullptr) {
      logp[r] = 0.f;
      lse[r] = 0.f;
    }
    if (token_loss != nullptr) token_loss[r] = 0.f;
  }
  if (dhidden != nullptr) {
    float* dst = dhidden + r * lddh;
    for (int v = threadIdx.x; v < d; v += 256) dst[v] = 0.f;
  }
}

// loss = sum of the per-chunk shares, in chunk order.
__global__ void fopd_sum_chunks(const float* chunk_loss, int n, float* loss) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += static_cast<double>(chunk_loss[i]);
    loss[0] = static_cast<float>(s);
  }
}

}  // namespace fopd

#endif  // FOPD_GEMM_HIP_
