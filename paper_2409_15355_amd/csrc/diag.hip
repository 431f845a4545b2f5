// Diagnostic for benchmarks, not on the hot path: the rate of v_mfma_f32_32x32x16_bf16 that the
// device sustains on operands with the bit activity of real data.  The attention core is priced
// against the nominal MFMA peak (2.4 GHz); a part that is power-limited on such data runs an MFMA
// loop well below that clock, and lower still when every MFMA is fed a fresh operand fragment from
// LDS, as the attention core's K and V fragments are.  This kernel measures exactly that: 8 waves per
// compute unit (two per SIMD), each issuing dependent-free MFMAs on four accumulators from a rolling
// window of eight operand fragments, of which 0, 1 or 2 per two MFMAs are re-read from LDS.
#include "ba_device.h"

namespace ba {
namespace {

constexpr int kDiagThreads = 512;
constexpr int kDiagLds = 128 * 1024;
constexpr int kDiagUnroll = 16;  // MFMAs per loop iteration

template <int READS_PER_TWO>
__global__ __launch_bounds__(kDiagThreads) void mfma_ceiling_kernel(unsigned long long *clocks, uint32_t *sink, int iters,
                                                                     uint32_t seed) {
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  typedef __attribute__((address_space(3))) char lds_c;
  typedef __attribute__((address_space(3))) u32x4_t lds_u32x4;
  lds_c *smem = (lds_c *)smem_generic;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // bf16 pairs with random signs and mantissas, magnitudes 1/4 .. 2
  uint32_t s = seed + threadIdx.x * 9781u + blockIdx.x * 6151u;
  auto draw = [&]() {
    s = s * 1664525u + 1013904223u;
    uint32_t h = s ^ (s >> 15);
    return (h & 0x80008000u) | 0x3e803e80u + ((h >> 3) & 0x01800180u) | ((h >> 9) & 0x007f007fu);
  };
  for (int i = threadIdx.x; i < kDiagLds / 4; i += kDiagThreads) ((__attribute__((address_space(3))) uint32_t *)smem)[i] = draw();
  __syncthreads();
  u32x4_t b[4], win[8];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) b[i][j] = draw();
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 4; ++j) win[i][j] = draw();
  f32x16_t acc[4];
  for (int i = 0; i < 4; ++i)
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  const uint32_t base = (uint32_t)wave * (kDiagLds / 8);
  const unsigned long long w0 = wall_clock64(), c0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kDiagUnroll; ++i) {
      // a fragment is requested seven MFMAs before its use, as in the attention core
      if (READS_PER_TWO == 2 || (READS_PER_TWO == 1 && (i & 1)))
        win[(i + 7) % 8] = *(lds_u32x4 *)(smem + base + i * 1024 + ((lane * 16 + it * 16) & 1008));
      acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, win[i % 8]),
                                                          __builtin_bit_cast(bf16x8_t, b[(i >> 2) & 3]), acc[i & 3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // keep the sums bounded (they would otherwise grow out of range and change the pipe's activity)
    if ((it & 63) == 63) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] *= 0.0009765625f;
    }
  }
  const unsigned long long c1 = clock64(), w1 = wall_clock64();
  uint32_t x = 0;
  for (int j = 0; j < 4; ++j)
    for (int v = 0; v < 16; ++v) x ^= __float_as_uint(acc[j][v]);
  if (lane == 0) {
    clocks[((size_t)blockIdx.x * 8 + wave) * 2] = c1 - c0;
    clocks[((size_t)blockIdx.x * 8 + wave) * 2 + 1] = w1 - w0;
  }
  sink[(size_t)blockIdx.x * kDiagThreads + threadIdx.x] = x;
}

}  // namespace

size_t diag_mfma_workspace_bytes(int n_wg) { return (size_t)n_wg * (8 * 2 * 8 + kDiagThreads * 4); }

hipError_t launch_mfma_ceiling(int reads_per_two, int n_wg, int iters, void *ws, uint32_t seed, hipStream_t stream) {
  unsigned long long *clocks = (unsigned long long *)ws;
  uint32_t *sink = (uint32_t *)((char *)ws + (size_t)n_wg * 8 * 2 * 8);
  const void *fn = reads_per_two == 0 ? (const void *)&mfma_ceiling_kernel<0>
                                      : reads_per_two == 1 ? (const void *)&mfma_ceiling_kernel<1> : (const void *)&mfma_ceiling_kernel<2>;
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kDiagLds);
  if (e != hipSuccess) return e;
  if (reads_per_two == 0)
    hipLaunchKernelGGL((mfma_ceiling_kernel<0>), dim3(n_wg), dim3(kDiagThreads), kDiagLds, stream, clocks, sink, iters, seed);
  else if (reads_per_two == 1)
    hipLaunchKernelGGL((mfma_ceiling_kernel<1>), dim3(n_wg), dim3(kDiagThreads), kDiagLds, stream, clocks, sink, iters, seed);
  else
    hipLaunchKernelGGL((mfma_ceiling_kernel<2>), dim3(n_wg), dim3(kDiagThreads), kDiagLds, stream, clocks, sink, iters, seed);
  return hipGetLastError();
}

}  // namespace ba
