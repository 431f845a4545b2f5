// Whole-prompt attention (Section 2.4) for fewer than four query heads per KV head.
//
// The short-block schedule packs the query heads of a KV group next to each other and is laid out
// for groups of four or more.  A smaller group G is run as a group of four: every KV head gets
// 4 - G phantom query heads whose rows are zero (a zero query has equal scores everywhere: a finite
// output that is never copied back; a zero output gradient adds nothing to dk and dv).  These two
// kernels move rows between the caller's [T][n_q_heads] tensors and the padded [T][4 n_kv_heads]
// ones.  Memory-bound copies of 16-byte chunks; the price of the route is the padded rows' share
// of the attention work, not these.
#include "ba_device.h"

namespace ba {
namespace {

constexpr int kPadThreads = 256;

// dst[t][kvh * GP + g] = g < G ? src[t][kvh * G + g] : 0, rows of `chunks` 16-byte pieces
__global__ __launch_bounds__(kPadThreads) void pad_heads_kernel(HeadPadParams p) {
  const int64_t n = p.tokens * p.n_kv_heads * p.group_padded * p.chunks;
  for (int64_t i = (int64_t)blockIdx.x * kPadThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kPadThreads) {
    const int c = (int)(i % p.chunks);
    int64_t r = i / p.chunks;
    const int g = (int)(r % p.group_padded);
    r /= p.group_padded;
    const int kvh = (int)(r % p.n_kv_heads);
    const int64_t t = r / p.n_kv_heads;
    const char *s = (const char *)p.real + (t * p.real_st + (int64_t)(kvh * p.group + (g < p.group ? g : 0)) * p.real_sh) * p.elt + c * 16;
    char *d = (char *)p.padded + (t * p.padded_st + (int64_t)(kvh * p.group_padded + g) * p.padded_sh) * p.elt + c * 16;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (g < p.group) v = *reinterpret_cast<const u32x4_t *>(s);
    *reinterpret_cast<u32x4_t *>(d) = v;
  }
}

// the way back: real[t][kvh * G + g] = padded[t][kvh * GP + g] for g < G
__global__ __launch_bounds__(kPadThreads) void unpad_heads_kernel(HeadPadParams p) {
  const int64_t n = p.tokens * p.n_kv_heads * p.group * p.chunks;
  for (int64_t i = (int64_t)blockIdx.x * kPadThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kPadThreads) {
    const int c = (int)(i % p.chunks);
    int64_t r = i / p.chunks;
    const int g = (int)(r % p.group);
    r /= p.group;
    const int kvh = (int)(r % p.n_kv_heads);
    const int64_t t = r / p.n_kv_heads;
    char *d = (char *)p.real + (t * p.real_st + (int64_t)(kvh * p.group + g) * p.real_sh) * p.elt + c * 16;
    const char *s = (const char *)p.padded + (t * p.padded_st + (int64_t)(kvh * p.group_padded + g) * p.padded_sh) * p.elt + c * 16;
    *reinterpret_cast<u32x4_t *>(d) = *reinterpret_cast<const u32x4_t *>(s);
  }
}

// log-sum-exps, one float per (token, head): the same two moves on 4-byte elements
__global__ __launch_bounds__(kPadThreads) void pad_lse_kernel(float *real, float *padded, int64_t tokens,
                                                              int n_kv_heads, int group, int group_padded, int to_padded) {
  const int gq = to_padded ? group_padded : group;
  const int64_t n = tokens * n_kv_heads * gq;
  for (int64_t i = (int64_t)blockIdx.x * kPadThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kPadThreads) {
    const int g = (int)(i % gq);
    const int64_t r = i / gq;
    const int kvh = (int)(r % n_kv_heads);
    const int64_t t = r / n_kv_heads;
    const int64_t ri = (t * n_kv_heads + kvh) * group + (g < group ? g : 0), pi = (t * n_kv_heads + kvh) * group_padded + g;
    if (to_padded) padded[pi] = g < group ? real[ri] : 0.f;
    else real[ri] = padded[pi];
  }
}

// Pseudo-random bf16 values of magnitude 1/8 .. 2 with random signs and mantissas (a hash of the
// element index): synthetic operands for the speed probe.
__global__ __launch_bounds__(kPadThreads) void fill_random_bf16_kernel(uint16_t *dst, int64_t n, uint32_t seed) {
  for (int64_t i = (int64_t)blockIdx.x * kPadThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kPadThreads) {
    uint32_t h = (uint32_t)i * 0x9e3779b1u + seed;
    h ^= h >> 16;
    h *= 0x7feb352du;
    h ^= h >> 15;
    h *= 0x846ca68bu;
    h ^= h >> 16;
    const uint32_t sign = (h >> 31) << 15, expo = (124u + ((h >> 8) & 3u)) << 7, mant = h & 0x7fu;
    dst[i] = (uint16_t)(sign | expo | mant);
  }
}

unsigned grid_for(int64_t n) {
  const int64_t wg = (n + kPadThreads - 1) / kPadThreads;
  return (unsigned)(wg < 1 ? 1 : (wg > 8192 ? 8192 : wg));
}

}  // namespace

hipError_t launch_pad_heads(const HeadPadParams &p, bool to_padded, hipStream_t stream) {
  if (p.tokens <= 0) return hipSuccess;
  const int64_t n = p.tokens * p.n_kv_heads * (to_padded ? p.group_padded : p.group) * p.chunks;
  if (to_padded)
    hipLaunchKernelGGL(pad_heads_kernel, dim3(grid_for(n)), dim3(kPadThreads), 0, stream, p);
  else
    hipLaunchKernelGGL(unpad_heads_kernel, dim3(grid_for(n)), dim3(kPadThreads), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_fill_random_bf16(uint16_t *dst, int64_t n, uint32_t seed, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_random_bf16_kernel, dim3(grid_for(n)), dim3(kPadThreads), 0, stream, dst, n, seed);
  return hipGetLastError();
}

hipError_t launch_pad_lse(float *real, float *padded, int64_t tokens, int n_kv_heads, int group, int group_padded,
                          bool to_padded, hipStream_t stream) {
  if (tokens <= 0) return hipSuccess;
  const int64_t n = tokens * n_kv_heads * (to_padded ? group_padded : group);
  hipLaunchKernelGGL(pad_lse_kernel, dim3(grid_for(n)), dim3(kPadThreads), 0, stream, real, padded, tokens, n_kv_heads,
                     group, group_padded, to_padded ? 1 : 0);
  return hipGetLastError();
}

}  // namespace ba
