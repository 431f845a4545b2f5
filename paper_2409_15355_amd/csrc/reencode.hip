// Position re-encoding of cached keys (Section 2.3 of arXiv 2409.15355): the two
// rotations of Eq. 2 and Eq. 3 collapse into one rotation by the position difference,
// applied here as a single coalesced HBM pass: 16-byte loads, fp32 rotate, 16-byte
// stores.  Memory-bound: 2 B read + 2 B written per bf16 element.
//
// Thread mapping.  A head vector of D elements is CH = D / VEC 16-byte chunks.  A
// thread owns chunk c and chunk c + CH/2 of one token and walks over that token's KV
// heads, so its VEC (cos, sin) pairs are computed once per token (ABSOLUTE mode) or
// once per workgroup (SHIFT mode: the angle depends on the block only) and reused for
// every head.  CH/2 neighbouring lanes cover half a head vector contiguously.
#include "ba_device.h"

namespace ba {
namespace {

constexpr int kThreads = 256;

template <typename T>
struct Chunk;  // 16 bytes of T as floats

template <>
struct Chunk<uint16_t> {
  static constexpr int VEC = 8;
  float f[8];
  __device__ __forceinline__ void load(const uint16_t *p) {
    u32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = bf16_lo(w[i]);
      f[2 * i + 1] = bf16_hi(w[i]);
    }
  }
  __device__ __forceinline__ void store(uint16_t *p) const {
    u32x4_t w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack_bf16(f[2 * i], f[2 * i + 1]);
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t *>(p));
  }
};

template <>
struct Chunk<float> {
  static constexpr int VEC = 4;
  float f[4];
  __device__ __forceinline__ void load(const float *p) {
    f32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = w[i];
  }
  __device__ __forceinline__ void store(float *p) const {
    f32x4_t w = {f[0], f[1], f[2], f[3]};
    __builtin_nontemporal_store(w, reinterpret_cast<f32x4_t *>(p));
  }
};

// y = R(angle) x on one (a, b) pair: [[c, -s], [s, c]] (Eq. 1 / Eq. 3).
__device__ __forceinline__ void rotate(float &a, float &b, float c, float s) {
  float na = c * a - s * b;
  float nb = s * a + c * b;
  a = na;
  b = nb;
}

template <typename T, int D, int LAYOUT, int MODE, int TOK_PER_WG, typename Blocks>
__global__ __launch_bounds__(kThreads) void reencode_kernel(ReencParams p, Blocks blocks, RopeTable rt) {
  constexpr int VEC = Chunk<T>::VEC;
  constexpr int CH = D / VEC;           // chunks per head vector
  constexpr int TPV = CH / 2;           // threads per head vector
  constexpr int TPP = kThreads / TPV;   // tokens per pass
  static_assert(TOK_PER_WG % TPP == 0, "tokens per workgroup must be whole passes");

  const int b = blockIdx.y;
  const int layer = blockIdx.z;
  const int len = blocks.len[b];
  // blockIdx.x = token chunk * head groups + head group: small inputs spread their heads over
  // more workgroups, large ones keep all heads in one thread so that sin/cos are reused
  const int hg = blockIdx.x % p.n_head_groups;
  const int tok0 = (blockIdx.x / p.n_head_groups) * TOK_PER_WG;
  if (tok0 >= len) return;

  const int c = threadIdx.x % TPV;
  const int tl = threadIdx.x / TPV;

  // frequencies of this thread's VEC pairs
  uint64_t turns[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    int j;
    if (LAYOUT == 0)  // interleaved: pairs live inside each chunk
      j = (e < VEC / 2) ? c * (VEC / 2) + e : (c + CH / 2) * (VEC / 2) + (e - VEC / 2);
    else  // half: element e of chunk c pairs with element e of chunk c + CH/2
      j = c * VEC + e;
    turns[e] = rt.turns[j];
  }

  const int shift0 = layer >= p.copy_from_layer ? 0 : blocks.pos_new[b] - blocks.pos_old[b];
  const T *src = static_cast<const T *>(p.src) + (int64_t)layer * p.src_sl +
                 (int64_t)blocks.src_off[b] * p.src_st;
  T *dst = static_cast<T *>(p.dst) + (int64_t)layer * p.dst_sl + (int64_t)blocks.dst_off[b] * p.dst_st;

  float cs[VEC], sn[VEC];
  if (MODE == 0) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) sincos_phase(rope_phase(shift0, turns[e]), cs[e], sn[e]);
  }
  // zero shift, or a layer that only rides along: bit-for-bit copy
  const bool plain_copy = ((MODE == 0) && (shift0 == 0)) || layer >= p.copy_from_layer;
  const int g_begin = hg * p.heads_per_thread;
  const int g_end = min(p.n_kv_heads, g_begin + p.heads_per_thread);

#pragma unroll 1
  for (int pass = 0; pass < TOK_PER_WG / TPP; ++pass) {
    const int u = tok0 + pass * TPP + tl;
    if (u >= len) break;
    if (MODE == 1) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) sincos_phase(rope_phase(shift0 + u, turns[e]), cs[e], sn[e]);
    }
    const T *s0 = src + (int64_t)u * p.src_st + c * VEC;
    T *d0 = dst + (int64_t)u * p.dst_st + c * VEC;
#pragma unroll 4
    for (int g = g_begin; g < g_end; ++g) {
      Chunk<T> x, y;
      x.load(s0 + g * p.src_sh);
      y.load(s0 + g * p.src_sh + (CH / 2) * VEC);
      if (!plain_copy) {
        if (LAYOUT == 0) {
#pragma unroll
          for (int e = 0; e < VEC / 2; ++e) {
            rotate(x.f[2 * e], x.f[2 * e + 1], cs[e], sn[e]);
            rotate(y.f[2 * e], y.f[2 * e + 1], cs[VEC / 2 + e], sn[VEC / 2 + e]);
          }
        } else {
#pragma unroll
          for (int e = 0; e < VEC; ++e) rotate(x.f[e], y.f[e], cs[e], sn[e]);
        }
      }
      x.store(d0 + g * p.dst_sh);
      y.store(d0 + g * p.dst_sh + (CH / 2) * VEC);
    }
  }
}

// Fast path: uniform shift (the angle depends on the block only), interleaved pairs (every pair
// lives inside one 16-byte chunk) and packed [tokens][heads][D] storage.  A block is then one
// contiguous run of chunks, and because the workgroup size is a multiple of the chunks per head
// vector, a thread that walks the run with stride 256 always meets the same four frequencies:
// a pure streaming pass, every wave instruction moving 1 KB of consecutive memory.
template <typename T, int D, int UNROLL, typename Blocks>
__global__ __launch_bounds__(kThreads) void reencode_shift_linear_kernel(ReencParams p, Blocks blocks, RopeTable rt) {
  constexpr int VEC = Chunk<T>::VEC;
  constexpr int CH = D / VEC;
  static_assert(kThreads % CH == 0, "a thread must keep its chunk position inside the head vector");
  const int b = blockIdx.y;
  const int layer = blockIdx.z;
  const int64_t n_chunks = (int64_t)blocks.len[b] * p.n_kv_heads * CH;
  const int64_t first = (int64_t)blockIdx.x * (UNROLL * kThreads) + threadIdx.x;
  if ((int64_t)blockIdx.x * (UNROLL * kThreads) >= n_chunks) return;
  const int c = threadIdx.x % CH;
  const int shift0 = layer >= p.copy_from_layer ? 0 : blocks.pos_new[b] - blocks.pos_old[b];
  float cs[VEC / 2], sn[VEC / 2];
#pragma unroll
  for (int e = 0; e < VEC / 2; ++e) sincos_phase(rope_phase(shift0, rt.turns[c * (VEC / 2) + e]), cs[e], sn[e]);
  const T *src = static_cast<const T *>(p.src) + (int64_t)layer * p.src_sl + (int64_t)blocks.src_off[b] * p.src_st;
  T *dst = static_cast<T *>(p.dst) + (int64_t)layer * p.dst_sl + (int64_t)blocks.dst_off[b] * p.dst_st;
  Chunk<T> x[UNROLL];
#pragma unroll
  for (int k = 0; k < UNROLL; ++k) {
    const int64_t L = first + (int64_t)k * kThreads;
    if (L < n_chunks) x[k].load(src + L * VEC);
  }
  if (shift0 != 0) {  // zero shift: bit-for-bit copy
#pragma unroll
    for (int k = 0; k < UNROLL; ++k)
#pragma unroll
      for (int e = 0; e < VEC / 2; ++e) rotate(x[k].f[2 * e], x[k].f[2 * e + 1], cs[e], sn[e]);
  }
#pragma unroll
  for (int k = 0; k < UNROLL; ++k) {
    const int64_t L = first + (int64_t)k * kThreads;
    if (L < n_chunks) x[k].store(dst + L * VEC);
  }
}

template <typename T, int D, typename Blocks>
hipError_t launch_linear(const ReencParams &p, const Blocks &blocks, const RopeTable &rt, hipStream_t stream) {
  constexpr int UNROLL = 8;
  constexpr int CH = D / Chunk<T>::VEC;
  const int64_t max_chunks = (int64_t)p.max_len * p.n_kv_heads * CH;
  dim3 grid((unsigned)((max_chunks + UNROLL * kThreads - 1) / (UNROLL * kThreads)), blocks.n, p.n_layers);
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return hipSuccess;
  hipLaunchKernelGGL((reencode_shift_linear_kernel<T, D, UNROLL, Blocks>), grid, dim3(kThreads), 0, stream, p, blocks, rt);
  return hipGetLastError();
}

template <typename T, int D, int LAYOUT, int MODE, typename Blocks>
hipError_t launch_t(const ReencParams &p, const Blocks &blocks, const RopeTable &rt, hipStream_t stream) {
  constexpr int VEC = Chunk<T>::VEC;
  constexpr int TPP = kThreads / (D / VEC / 2);
  constexpr int TOK_PER_WG = TPP;
  dim3 grid(((p.max_len + TOK_PER_WG - 1) / TOK_PER_WG) * p.n_head_groups, blocks.n, p.n_layers);
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return hipSuccess;
  hipLaunchKernelGGL((reencode_kernel<T, D, LAYOUT, MODE, TOK_PER_WG, Blocks>), grid, dim3(kThreads), 0,
                     stream, p, blocks, rt);
  return hipGetLastError();
}

template <typename T, int D, typename Blocks>
hipError_t launch_d(const ReencParams &p, const Blocks &blocks, const RopeTable &rt, hipStream_t stream) {
  const bool packed = p.src_sh == D && p.dst_sh == D && p.src_st == (int64_t)p.n_kv_heads * D &&
                      p.dst_st == (int64_t)p.n_kv_heads * D;
  if (p.layout == 0 && p.mode == 0 && packed) return launch_linear<T, D>(p, blocks, rt, stream);
  if (p.layout == 0)
    return p.mode == 0 ? launch_t<T, D, 0, 0>(p, blocks, rt, stream)
                       : launch_t<T, D, 0, 1>(p, blocks, rt, stream);
  return p.mode == 0 ? launch_t<T, D, 1, 0>(p, blocks, rt, stream)
                     : launch_t<T, D, 1, 1>(p, blocks, rt, stream);
}

}  // namespace

template <typename Blocks>
hipError_t launch_reencode_any(const ReencParams &p, const Blocks &blocks, const RopeTable &rt, hipStream_t stream) {
  if (p.dtype == 0) {
    if (p.head_dim == 128) return launch_d<uint16_t, 128>(p, blocks, rt, stream);
    if (p.head_dim == 64) return launch_d<uint16_t, 64>(p, blocks, rt, stream);
  } else {
    if (p.head_dim == 128) return launch_d<float, 128>(p, blocks, rt, stream);
    if (p.head_dim == 64) return launch_d<float, 64>(p, blocks, rt, stream);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_reencode(const ReencParams &p, const ReencBlocks &blocks, const RopeTable &rt, hipStream_t stream) {
  return launch_reencode_any(p, blocks, rt, stream);
}
hipError_t launch_reencode(const ReencParams &p, const ReencBlocksLarge &blocks, const RopeTable &rt,
                           hipStream_t stream) {
  return launch_reencode_any(p, blocks, rt, stream);
}

}  // namespace ba
