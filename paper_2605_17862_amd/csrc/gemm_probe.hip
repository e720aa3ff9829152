// Timing of the bf16 contraction kernel and of its bound-analysis variants on one shape.
//
//   gemm_probe [N rows, default 8192] [M, default 151936] [K, default 4096] [row padding in elements, default 0]
//              [groups of 20 back-to-back launches of the shipped loop, default 3] [operand values: 0 (default)
//              magnitudes in [0.5, 1), 1 close to normal with the spread of hidden states and projection weights]
//
// Out[N, M] = Bn[N, K] . Am[M, K]^T with fopd_gemm_nt (the kernel behind the three contractions of the loss pass
// through the projection; its main loop is that of the projection kernel fused with the log-sum-exp).  Prints,
// for the shipped wavefront shape and for the alternative one, the rate of the whole loop and of four variants
// that each leave one part of the loop out (their results are wrong on purpose): all global loads hitting the
// L1, no global loads, no LDS reads, matrix cores only.  (Tiles wider than 256 x 256 -- 256 x 320, 256 x 384 with
// four wavefronts -- need more than 256 accumulator registers per lane; hipcc spills 236 .. 712 registers per
// lane for them, so they are not built.)
// Under `rocprofv3 --pmc ...` the same program gives the counters of each variant.

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "fopd_gemm.hip"

#define CHECK(x)                                                                     \
  do {                                                                               \
    hipError_t e_ = (x);                                                             \
    if (e_ != hipSuccess) {                                                          \
      fprintf(stderr, "gemm_probe: %s failed: %s\n", #x, hipGetErrorString(e_));     \
      return 1;                                                                      \
    }                                                                                \
  } while (0)

__device__ inline uint32_t gemm_probe_hash(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}

// normal == 0: bf16 values with magnitudes in [0.5, 1): random sign and mantissa, one exponent.
// normal != 0: close to N(0, scale^2) (a sum of 12 uniforms), the spread of the operands the pass sees: the
// rate the part sustains depends on the operand bits (more toggling, more power, a lower clock).
__global__ void gemm_probe_fill(uint16_t* p, size_t n, uint32_t seed, int normal, float scale) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n;
       i += static_cast<size_t>(gridDim.x) * blockDim.x) {
    if (normal == 0) {
      uint32_t h = static_cast<uint32_t>(i) * 2654435761u + seed;
      h ^= h >> 15;
      p[i] = static_cast<uint16_t>(((h & 1u) << 15) | (0x3f00u + ((h >> 8) & 0x7fu)));
    } else {
      float acc = 0.f;
      for (uint32_t k = 0; k < 12u; ++k)
        acc += static_cast<float>(gemm_probe_hash(static_cast<uint32_t>(i) * 12u + k + seed * 0x9e3779b9u) >> 8) *
               (1.0f / 16777216.0f);
      p[i] = static_cast<uint16_t>(__float_as_uint((acc - 6.0f) * scale) >> 16);
    }
  }
}

template <int PROBE, int WM, int WN, int TJ, int VIA_REGS>
static int run(const char* name, const __bf16* A, int64_t lda, int M, const __bf16* B, int64_t ldb, int N, int K,
               float* out, hipEvent_t e0, hipEvent_t e1) {
  using namespace fopd;
  auto kern = fopd_gemm_nt<false, PROBE, WM, WN, TJ, VIA_REGS>;
  constexpr int lds = gemm_lds_bytes(WN, TJ), tn = gemm_tile_n(WN, TJ);
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds) !=
      hipSuccess) {
    (void)hipGetLastError();
    printf("gemm_probe: %-34s not runnable: %d bytes of LDS refused\n", name, lds);
    return 0;
  }
  const int tiles_m = (M + kGemmTile - 1) / kGemmTile, tiles_n = (N + tn - 1) / tn;
  const unsigned grid = static_cast<unsigned>(((tiles_m + 7) / 8) * ((tiles_n + 31) / 32) * 256);
  float total = 0.f;
  for (int rep = 0; rep < 4; ++rep) {          // first launch is a warm-up
    CHECK(hipEventRecord(e0, 0));
    kern<<<grid, 64 * WM * WN, lds>>>(A, lda, M, B, ldb, N, K, out, M, tiles_m, tiles_n, nullptr);
    CHECK(hipGetLastError());
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    if (rep > 0) total += ms;
  }
  const double flops = 2.0 * M * static_cast<double>(N) * K;
  printf("gemm_probe: %-34s avg %.3f ms, %.0f TFLOP/s (%.3f of 2500)\n", name, total / 3, flops / (total / 3) * 1e-9,
         flops / (total / 3) * 1e-9 / 2500.0);
  fflush(stdout);
  return 0;
}

// The shipped loop launched back to back, with no idle time between launches: the rate the part sustains, as
// inside a pass that runs contractions for hundreds of milliseconds.  Groups of 20 launches, timed apiece.
static int run_sustained(const __bf16* A, int64_t lda, int M, const __bf16* B, int64_t ldb, int N, int K, float* out,
                         int groups, hipEvent_t e0, hipEvent_t e1) {
  using namespace fopd;
  auto kern = fopd_gemm_nt<false, 0, 2, 4, 2, 4>;
  constexpr int lds = gemm_lds_bytes(4, 2), tn = gemm_tile_n(4, 2);
  CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  const int tiles_m = (M + kGemmTile - 1) / kGemmTile, tiles_n = (N + tn - 1) / tn;
  const unsigned grid = static_cast<unsigned>(((tiles_m + 7) / 8) * ((tiles_n + 31) / 32) * 256);
  const double flops = 2.0 * M * static_cast<double>(N) * K;
  for (int group = 0; group < groups; ++group) {
    CHECK(hipEventRecord(e0, 0));
    for (int rep = 0; rep < 20; ++rep) kern<<<grid, 512, lds>>>(A, lda, M, B, ldb, N, K, out, M, tiles_m, tiles_n, nullptr);
    CHECK(hipGetLastError());
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("gemm_probe: shipped loop, 20 launches back to back (group %d): avg %.3f ms, %.0f TFLOP/s (%.3f of 2500)\n",
           group, ms / 20, flops / (ms / 20) * 1e-9, flops / (ms / 20) * 1e-9 / 2500.0);
    fflush(stdout);
  }
  return 0;
}

int main(int argc, char** argv) {
  const int N = (argc > 1) ? atoi(argv[1]) : 8192;
  const int M = (argc > 2) ? atoi(argv[2]) : 151936;
  const int K = (argc > 3) ? atoi(argv[3]) : 4096;
  const int pad = (argc > 4) ? atoi(argv[4]) : 0;       // extra elements per operand row (row pitch K + pad)
  const int groups = (argc > 5) ? atoi(argv[5]) : 3;    // groups of 20 back-to-back launches of the shipped loop
  const int normal = (argc > 6) ? atoi(argv[6]) : 0;    // 1: operands close to N(0, 1) and N(0, (3/64)^2)
  if (N < 1 || N > 65536 || M < 4 || M > 262144 || M % 4 != 0 || K < 64 || K > 16384 || K % 64 != 0 || pad < 0 ||
      pad > 4096 || pad % 8 != 0 || groups < 0 || groups > 64) {
    fprintf(stderr, "gemm_probe: N in [1, 65536], M in [4, 262144] and a multiple of 4, K a multiple of 64 in [64, 16384]\n");
    return 2;
  }
  __bf16 *A = nullptr, *B = nullptr;
  float* out = nullptr;
  const int64_t ld = K + pad;
  CHECK(hipMalloc(&A, static_cast<size_t>(M) * ld * 2));
  CHECK(hipMalloc(&B, static_cast<size_t>(N) * ld * 2));
  CHECK(hipMalloc(&out, static_cast<size_t>(N) * M * 4));
  gemm_probe_fill<<<4096, 256>>>(reinterpret_cast<uint16_t*>(A), static_cast<size_t>(M) * ld, 1u, normal, 0.046875f);
  gemm_probe_fill<<<4096, 256>>>(reinterpret_cast<uint16_t*>(B), static_cast<size_t>(N) * ld, 2u, normal, 1.0f);
  CHECK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  printf("gemm_probe: Out[%d, %d] = Bn[%d, %d] . Am[%d, %d]^T, bf16 in, fp32 out, operand row pitch %ld elements, %s\n", N,
         M, N, K, M, K, static_cast<long>(ld),
         normal ? "operands close to N(0, 1) and N(0, (3/64)^2)" : "operand magnitudes in [0.5, 1)");
#define FOPD_PROBE_SET(WM, WN, TJ)                                                                  \
  if (run<0, WM, WN, TJ, 0>("whole loop, direct global -> LDS loads", A, ld, M, B, ld, N, K, out, e0, e1)) return 1; \
  if (run<1, WM, WN, TJ, 0>("all global loads hit the L1", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;            \
  if (run<2, WM, WN, TJ, 0>("no global loads", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;                        \
  if (run<3, WM, WN, TJ, 0>("no LDS reads", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;                           \
  if (run<4, WM, WN, TJ, 0>("matrix cores only", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;                      \
  if (run<5, WM, WN, TJ, 0>("part of the n-side fill left out", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  printf("gemm_probe: tile 256 x 256, eight wavefronts of 128 x 64 (the shipped shape)\n");
  FOPD_PROBE_SET(2, 4, 2)
  if (run<0, 2, 4, 2, 1>("whole loop, stages through registers", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<0, 2, 4, 2, 2>("  ... n-side loads issued mid-pair", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<0, 2, 4, 2, 3>("  ... a quarter of the loads per slice", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<0, 2, 4, 2, 4>("  ... and of the LDS writes (shipped)", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<1, 2, 4, 2, 4>("  ... all global loads hit the L1", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<6, 2, 4, 2, 4>("  ... lines requested a pair ahead", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<7, 2, 4, 2, 4>("  ... wave priority raised for MFMAs", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<8, 2, 4, 2, 4>("  ... no result stores", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<9, 2, 4, 2, 4>("  ... non-temporal result stores", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<10, 2, 4, 2, 4>("  ... slice order left to the scheduler", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<11, 2, 4, 2, 4>("  ... fragment reads first in a slice", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<13, 2, 4, 2, 4>("  ... one memory instruction per gap", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<14, 2, 4, 2, 4>("  ... first round skewed by 512 cycles", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run_sustained(A, ld, M, B, ld, N, K, out, groups, e0, e1)) return 1;
  printf("gemm_probe: tile 256 x 256, four wavefronts of 128 x 128\n");
  FOPD_PROBE_SET(2, 2, 4)
  if (run<0, 2, 2, 4, 1>("whole loop, stages through registers", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
  if (run<0, 2, 2, 4, 4>("  ... a quarter of a pair per slice", A, ld, M, B, ld, N, K, out, e0, e1)) return 1;
#undef FOPD_PROBE_SET
  if (N >= 8192 && M == 151936 && K == 4096 && pad == 0) {
    // the weight gradient's shape with both operands k-major, in the same buffers: Out[151936, 4096] =
    // sum over 4096 rows of Bk[4096, 151936] (all of buffer A) and Ak[4096, 4096] (half of the first 8192 rows of
    // buffer B); three orders of the instructions inside a slice
    using namespace fopd;
    const int tm = 4096 / kGemmTile, tn = (151936 + kGemmTileN - 1) / kGemmTileN;
    const unsigned grid = static_cast<unsigned>(((tm + 7) / 8) * ((tn + 31) / 32) * 256);
    const double flops = 2.0 * 4096 * 151936.0 * 4096;
    auto time_tn = [&](auto kern, const char* name) -> int {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              kTnLdsBytes) != hipSuccess) {
        printf("gemm_probe: %d bytes of LDS refused\n", kTnLdsBytes);
        return 1;
      }
      float total = 0.f;
      for (int rep = 0; rep < 4; ++rep) {
        CHECK(hipEventRecord(e0, 0));
        kern<<<grid, kGemmThreads, kTnLdsBytes>>>(B, 4096, 4096, 4096, A, 151936, 151936, 4096, out, 4096, tm, tn, nullptr);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0.f;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (rep > 0) total += ms;
      }
      printf("gemm_probe: both operands k-major, Out[151936, 4096], K = 4096, %s: avg %.3f ms, %.0f TFLOP/s (%.3f of 2500)\n",
             name, total / 3, flops / (total / 3) * 1e-9, flops / (total / 3) * 1e-9 / 2500.0);
      return 0;
    };
    if (time_tn(fopd_gemm_tn<false, 0>, "slice order left to the scheduler")) return 1;
    if (time_tn(fopd_gemm_tn<false, 1>, "reads four per gap")) return 1;
    if (time_tn(fopd_gemm_tn<false, 2>, "two memory instructions per gap (shipped)")) return 1;
  }
  CHECK(hipFree(A));
  CHECK(hipFree(B));
  CHECK(hipFree(out));
  return 0;
}
