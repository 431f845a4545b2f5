// Device-side helpers shared by the attention kernels: LDS-direct tile loads and the waits and
// barriers that go with them, the half-wave exchange, and the search in a table of tile starts.
#pragma once

#include "ba_device.h"

namespace ba {

__device__ __forceinline__ int find_segment(const int32_t *tile_start, int n, int tile) {
  int lo = 0, hi = n;  // largest i with tile_start[i] <= tile
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (tile_start[mid] <= tile) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ float other_half(float x) {
  // value held by lane ^ 32, combined with ours by the caller
  uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return (threadIdx.x & 32) ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}

typedef __attribute__((address_space(3))) char lds_char;

// LDS-direct load: every lane fetches 16 bytes from base + offset and the wave writes them to
// LDS bytes [lds_base + 16 lane, +16).  Issued through inline assembly ON PURPOSE: the compiler
// would otherwise treat the copy as a store that may alias every later LDS read and wait for
// it (vmcnt(0)) before the first fragment read of the same iteration, which exposes the whole
// HBM latency on every tile.  The price is that completion is ours to wait for: a dma_wait
// must come before the barrier that publishes the buffer.
__device__ __forceinline__ void lds_dma16(const char *base, uint32_t offset, uint32_t lds_base) {
  // base and lds_base are wave-uniform by construction; say so, or a value the compiler cannot
  // prove uniform would not fit the scalar operands
  const uint64_t b = (uint64_t)base;
  const uint64_t bu = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32)) << 32) |
                      (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  base = (const char *)bu;
  lds_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(offset), "s"(base), "s"(lds_base)
               : "memory");
}
// Wait until at most NEWER of this wave's vector-memory operations are still in flight
// (they complete in order), leaving the other counters alone.  gfx9 encoding of s_waitcnt.
// Workgroup barrier without the memory fence of __syncthreads(): LDS reads that are still in flight
// (fragments requested ahead of their use) need not drain first.  What a barrier publishes here are
// LDS-direct copies, and the copying wave has waited for those (dma_wait) before it arrives.
// (Written as assembly so that the compiler does not drain the LDS counter in front of it.)
__device__ __forceinline__ void wg_barrier() {
  asm volatile("s_barrier" ::: "memory");
}
template <int NEWER>
__device__ __forceinline__ void dma_wait() {
  static_assert(NEWER >= 0 && NEWER < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0f70 | (NEWER & 15) | ((NEWER >> 4) << 14));
  asm volatile("" ::: "memory");
}

}  // namespace ba
