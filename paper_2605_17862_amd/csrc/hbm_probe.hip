// Plain streaming kernels of known size: the yardstick for the loss pass.
//
//   hbm_probe [GiB per buffer, default 8]
//
// Times, five launches each after a warm-up, over buffers of the given size:
//   row shape (what the loss kernels use: one 256-lane workgroup per 303,872-byte row, 16-byte accesses)
//     read, write, copy
//   shapes that do NOT follow the loss kernels, as independent yardsticks for the same bytes
//     runtime copy      hipMemcpyAsync device-to-device (the runtime's own copy path)
//     flat copy         a fixed grid of 2048 workgroups striding over the buffer in 16 KB blocks
//     burst copy        each workgroup loads a 64 KB contiguous chunk into registers, then stores it
//     regs copy         one 1024-lane workgroup per compute unit walks rows, holding a whole row in registers
//                       between its loads and its stores (the shape of the row-in-registers loss kernel)
//     phased copy       the same, with every compute unit loading only in even and storing only in odd time slots of
//                       13 us of the chip's constant clock, so that the memory sees reads and writes in turn
//   read:write mixes, row shape
//     2r1w              two buffers read, one written (the mix of the two-tensor gradient kernel)
//     1r2w              one buffer read, two written
//     2r                two buffers read, nothing written (the two-tensor log-sum-exp kernel)
// and prints the bandwidth of each (bytes read + bytes written, over the time).  Under
// `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` the row-shape copy kernel gives the counter reading for a
// known number of bytes, which is the scale factor applied to the loss kernels' readings.

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kRowVecs = 18992;   // 151,936 bf16 = 303,872 bytes
constexpr int kFlatGrid = 2048;   // 8 workgroups per compute unit
constexpr int kBurst = 16;        // vectors per lane held in registers by the burst copy (64 KB per workgroup)

__global__ void __launch_bounds__(kThreads) hbm_probe_read(const u32x4* in, uint32_t* sink) {
  const u32x4* r = in + static_cast<size_t>(blockIdx.x) * kRowVecs;
  uint32_t acc = 0;
  int j = threadIdx.x;
  for (; j + 3 * kThreads < kRowVecs; j += 4 * kThreads) {     // four loads in flight per lane
    const u32x4 v0 = __builtin_nontemporal_load(r + j);
    const u32x4 v1 = __builtin_nontemporal_load(r + j + kThreads);
    const u32x4 v2 = __builtin_nontemporal_load(r + j + 2 * kThreads);
    const u32x4 v3 = __builtin_nontemporal_load(r + j + 3 * kThreads);
    acc ^= v0.x ^ v1.y ^ v2.z ^ v3.w;
  }
  for (; j < kRowVecs; j += kThreads) acc ^= __builtin_nontemporal_load(r + j).x;
  if (acc == 0x9e3779b9u) sink[0] = acc;   // never true for the fill pattern; keeps the loads alive
}

__global__ void __launch_bounds__(kThreads) hbm_probe_write(u32x4* out) {
  u32x4* o = out + static_cast<size_t>(blockIdx.x) * kRowVecs;
  const u32x4 v = {1u, 2u, 3u, blockIdx.x};
  for (int j = threadIdx.x; j < kRowVecs; j += kThreads) o[j] = v;
}

__global__ void __launch_bounds__(kThreads) hbm_probe_copy(const u32x4* in, u32x4* out) {
  const u32x4* r = in + static_cast<size_t>(blockIdx.x) * kRowVecs;
  u32x4* o = out + static_cast<size_t>(blockIdx.x) * kRowVecs;
  for (int j = threadIdx.x; j < kRowVecs; j += kThreads) o[j] = __builtin_nontemporal_load(r + j);
}

// n = total number of 16-byte vectors.  Block k of 1024 vectors goes to workgroup k % gridDim.
__global__ void __launch_bounds__(kThreads) hbm_probe_copy_flat(const u32x4* in, u32x4* out, size_t n) {
  const size_t step = static_cast<size_t>(gridDim.x) * 4 * kThreads;
  for (size_t base = static_cast<size_t>(blockIdx.x) * 4 * kThreads; base < n; base += step) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t i = base + u * kThreads + threadIdx.x;
      if (i < n) v[u] = __builtin_nontemporal_load(in + i);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t i = base + u * kThreads + threadIdx.x;
      if (i < n) __builtin_nontemporal_store(v[u], out + i);
    }
  }
}

__global__ void __launch_bounds__(kThreads) hbm_probe_copy_burst(const u32x4* in, u32x4* out, size_t n) {
  const size_t chunk = static_cast<size_t>(kBurst) * kThreads;
  const size_t step = static_cast<size_t>(gridDim.x) * chunk;
  for (size_t base = static_cast<size_t>(blockIdx.x) * chunk; base < n; base += step) {
    u32x4 v[kBurst];
#pragma unroll
    for (int u = 0; u < kBurst; ++u) {
      const size_t i = base + u * kThreads + threadIdx.x;
      if (i < n) v[u] = __builtin_nontemporal_load(in + i);
    }
#pragma unroll
    for (int u = 0; u < kBurst; ++u) {
      const size_t i = base + u * kThreads + threadIdx.x;
      if (i < n) __builtin_nontemporal_store(v[u], out + i);
    }
  }
}

__global__ void __launch_bounds__(kThreads) hbm_probe_2r1w(const u32x4* in1, const u32x4* in2, u32x4* out) {
  const size_t off = static_cast<size_t>(blockIdx.x) * kRowVecs;
  for (int j = threadIdx.x; j < kRowVecs; j += kThreads) {
    const u32x4 a = __builtin_nontemporal_load(in1 + off + j);
    const u32x4 b = __builtin_nontemporal_load(in2 + off + j);
    __builtin_nontemporal_store(a ^ b, out + off + j);
  }
}

// two buffers read row by row, nothing written (the shape of the two-tensor log-sum-exp kernel)
__global__ void __launch_bounds__(kThreads) hbm_probe_2r(const u32x4* in1, const u32x4* in2, uint32_t* sink) {
  const size_t off = static_cast<size_t>(blockIdx.x) * kRowVecs;
  uint32_t acc = 0;
  int j = threadIdx.x;
  for (; j + kThreads < kRowVecs; j += 2 * kThreads) {       // two loads of each buffer in flight per lane
    const u32x4 a0 = __builtin_nontemporal_load(in1 + off + j);
    const u32x4 b0 = __builtin_nontemporal_load(in2 + off + j);
    const u32x4 a1 = __builtin_nontemporal_load(in1 + off + j + kThreads);
    const u32x4 b1 = __builtin_nontemporal_load(in2 + off + j + kThreads);
    acc ^= a0.x ^ b0.y ^ a1.z ^ b1.w;
  }
  for (; j < kRowVecs; j += kThreads)
    acc ^= __builtin_nontemporal_load(in1 + off + j).x ^ __builtin_nontemporal_load(in2 + off + j).y;
  if (acc == 0x9e3779b9u) sink[0] = acc;   // never true for the fill patterns; keeps the loads alive
}

__global__ void __launch_bounds__(kThreads) hbm_probe_1r2w(const u32x4* in, u32x4* out1, u32x4* out2) {
  const size_t off = static_cast<size_t>(blockIdx.x) * kRowVecs;
  for (int j = threadIdx.x; j < kRowVecs; j += kThreads) {
    const u32x4 a = __builtin_nontemporal_load(in + off + j);
    __builtin_nontemporal_store(a, out1 + off + j);
    __builtin_nontemporal_store(~a, out2 + off + j);
  }
}

#define CHECK(x)                                                                    \
  do {                                                                              \
    hipError_t e_ = (x);                                                            \
    if (e_ != hipSuccess) {                                                         \
      fprintf(stderr, "hbm_probe: %s failed: %s\n", #x, hipGetErrorString(e_));     \
      return 1;                                                                     \
    }                                                                               \
  } while (0)

constexpr int kRegsThreads = 1024, kRegsVecs = (kRowVecs + kRegsThreads - 1) / kRegsThreads;

// Leaves as soon as the constant 100 MHz clock is in a slot of the wanted kind (slots of `slot` ticks; even ones are
// for loads, odd ones for stores).  The clock advances, so every wavefront leaves.
__device__ __forceinline__ void hbm_probe_wait_slot(unsigned want_odd, unsigned slot) {
  for (;;) {
    const unsigned long long t = __builtin_amdgcn_s_memrealtime();
    if (static_cast<unsigned>((t / slot) & 1ull) == want_odd) break;
    __builtin_amdgcn_s_sleep(2);
  }
}

// slot = 0: loads and stores of the compute units fall as they come; else: see above.
__global__ void __launch_bounds__(kRegsThreads) hbm_probe_copy_regs(const u32x4* in, u32x4* out, int rows, unsigned slot) {
  u32x4 v[kRegsVecs];
  for (int row = blockIdx.x; row < rows; row += gridDim.x) {
    const u32x4* r = in + static_cast<size_t>(row) * kRowVecs;
    u32x4* o = out + static_cast<size_t>(row) * kRowVecs;
    if (slot != 0) hbm_probe_wait_slot(0, slot);
#pragma unroll
    for (int k = 0; k < kRegsVecs; ++k) {
      const int j = threadIdx.x + k * kRegsThreads;
      if (j < kRowVecs) v[k] = __builtin_nontemporal_load(r + j);
    }
    if (slot != 0) hbm_probe_wait_slot(1, slot);
#pragma unroll
    for (int k = 0; k < kRegsVecs; ++k) {
      const int j = threadIdx.x + k * kRegsThreads;
      if (j < kRowVecs) __builtin_nontemporal_store(v[k], o + j);
    }
  }
}

int main(int argc, char** argv) {
  const double gib = (argc > 1) ? atof(argv[1]) : 8.0;
  if (!(gib > 0.0) || gib > 64.0) {
    fprintf(stderr, "hbm_probe: size must be in (0, 64] GiB\n");
    return 2;
  }
  const size_t row_bytes = static_cast<size_t>(kRowVecs) * 16;
  const unsigned rows = static_cast<unsigned>(gib * 1073741824.0 / row_bytes);
  const size_t bytes = rows * row_bytes;
  const size_t nvec = static_cast<size_t>(rows) * kRowVecs;
  u32x4 *a = nullptr, *b = nullptr, *c = nullptr;
  uint32_t* sink = nullptr;
  CHECK(hipMalloc(&a, bytes));
  CHECK(hipMalloc(&b, bytes));
  CHECK(hipMalloc(&c, bytes));
  CHECK(hipMalloc(&sink, 4));
  CHECK(hipMemset(a, 1, bytes));
  CHECK(hipMemset(b, 2, bytes));
  CHECK(hipMemset(c, 3, bytes));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  printf("hbm_probe: %u rows of %zu bytes = %.3f GB per buffer\n", rows, row_bytes, bytes * 1e-9);
  const char* names[11] = {"read", "write", "copy", "runtime-copy", "flat-copy", "burst-copy", "2r1w", "1r2w", "2r",
                           "regs-copy", "phased-copy"};
  const double factor[11] = {1.0, 1.0, 2.0, 2.0, 2.0, 2.0, 3.0, 3.0, 2.0, 2.0, 2.0};
  int cus = 256;
  {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, 0) == hipSuccess && prop.multiProcessorCount > 0) cus = prop.multiProcessorCount;
  }
  for (int which = 0; which < 11; ++which) {
    const double moved = factor[which] * bytes;
    float total = 0.f;
    for (int rep = 0; rep < 6; ++rep) {        // first launch is a warm-up
      CHECK(hipEventRecord(e0, 0));
      switch (which) {
        case 0: hbm_probe_read<<<rows, kThreads>>>(a, sink); break;
        case 1: hbm_probe_write<<<rows, kThreads>>>(b); break;
        case 2: hbm_probe_copy<<<rows, kThreads>>>(a, b); break;
        case 3: CHECK(hipMemcpyAsync(b, a, bytes, hipMemcpyDeviceToDevice, 0)); break;
        case 4: hbm_probe_copy_flat<<<kFlatGrid, kThreads>>>(a, b, nvec); break;
        case 5: hbm_probe_copy_burst<<<kFlatGrid, kThreads>>>(a, b, nvec); break;
        case 6: hbm_probe_2r1w<<<rows, kThreads>>>(a, c, b); break;
        case 7: hbm_probe_1r2w<<<rows, kThreads>>>(a, b, c); break;
        case 8: hbm_probe_2r<<<rows, kThreads>>>(a, c, sink); break;
        case 9: hbm_probe_copy_regs<<<cus, kRegsThreads>>>(a, b, static_cast<int>(rows), 0u); break;
        default: hbm_probe_copy_regs<<<cus, kRegsThreads>>>(a, b, static_cast<int>(rows), 1300u); break;
      }
      CHECK(hipGetLastError());
      CHECK(hipEventRecord(e1, 0));
      CHECK(hipEventSynchronize(e1));
      float ms = 0.f;
      CHECK(hipEventElapsedTime(&ms, e0, e1));
      if (rep > 0) total += ms;
    }
    printf("hbm_probe: %-12s %.0f bytes per launch, avg %.3f ms, %.0f GB/s\n", names[which], moved, total / 5,
           moved / (total / 5) * 1e-6);
    fflush(stdout);
  }
  CHECK(hipFree(a));
  CHECK(hipFree(b));
  CHECK(hipFree(c));
  CHECK(hipFree(sink));
  return 0;
}
