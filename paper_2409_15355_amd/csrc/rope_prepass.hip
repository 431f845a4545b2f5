// RoPE pre-pass for fresh queries and keys (Eq. 1 of arXiv 2409.15355, positions per
// Section 2.3: local to the block for per-block encoding, absolute for the final block).
//
// One launch rotates the un-rotated K rows (the result is the cacheable key, an output of the
// step anyway) and the Q rows of a run of segments; Q is also multiplied by
// softmax_scale * log2(e) before its one rounding to bf16, so that the attention core's
// score accumulators hold base-2 exponents directly.  Doing this ahead of the attention core
// keeps 32 sin/cos evaluations per lane out of every workgroup's start-up.
//
// Thread mapping as in the re-encode kernel: a thread owns 16-byte chunk c and chunk c + CH/2
// of one token and walks a group of heads, its sin/cos computed once.  Few tokens: one head
// per thread (many short threads); many tokens: several heads per thread.
#include <string.h>

#include <algorithm>

#include "ba_device.h"

namespace ba {
namespace {

constexpr int kThreads = 256;

// Table of rotations for the block-table form of the final block: row b, frequency j holds
// (cos, sin) of angle[b] * theta_j.  One thread per entry.
template <int NB>
__global__ __launch_bounds__(kThreads) void rope_rot_table_kernel(float *dst, int n_rot, int half_dim,
                                                                  RopeRotsT<NB> rots, RopeTable rt) {
  const int idx = blockIdx.x * kThreads + threadIdx.x;
  if (idx >= n_rot * half_dim) return;
  const int b = idx / half_dim, j = idx - b * half_dim;
  float c, s;
  sincos_phase(rope_phase(rots.angle[b], rt.turns[j]), c, s);
  reinterpret_cast<float2 *>(dst)[idx] = make_float2(c, s);
}

// workgroup rows of the Q job: head groups, or one row when only the table of factors is written
__host__ __device__ inline int q_groups(const RopePrepassParams &p) {
  return (p.do_q == 1 || p.do_q == 3) ? (p.n_q_heads + p.heads_per_thread - 1) / p.heads_per_thread
                                      : ((p.do_q == 2 || p.do_q == 4) ? 1 : 0);
}

template <int D, int LAYOUT, typename Segs>
__global__ __launch_bounds__(kThreads) void rope_prepass_kernel(RopePrepassParams p, Segs segs, RopeTable rt,
                                                                RopeRotsSmall rots) {
  constexpr int VEC = 8;
  constexpr int CH = D / VEC;
  constexpr int TPV = CH / 2;          // threads per head vector
  constexpr int TPP = kThreads / TPV;  // tokens per workgroup
  {
    // workgroup rows beyond the head groups fill a (small) table of rotations, one thread per entry
    const int head_groups = q_groups(p) + (p.do_k ? (p.n_kv_heads + p.heads_per_thread - 1) / p.heads_per_thread : 0);
    if ((int)blockIdx.y >= head_groups) {
      const int idx = (((int)blockIdx.y - head_groups) * (int)gridDim.x + (int)blockIdx.x) * kThreads + (int)threadIdx.x;
      if (idx < p.n_rot * (D / 2)) {
        const int b = idx / (D / 2), j = idx - b * (D / 2);
        float c, s;
        sincos_phase(rope_phase(rots.angle[b], rt.turns[j]), c, s);
        reinterpret_cast<float2 *>(p.rot_dst)[idx] = make_float2(c, s);
      }
      return;
    }
  }
  const int c = threadIdx.x % TPV;
  // which tensor and which heads this workgroup handles: Q head groups first, then K
  const int groups_q = q_groups(p);
  const bool is_q = (int)blockIdx.y < groups_q;
  int t = segs.start[0] + blockIdx.x * TPP + threadIdx.x / TPV;
  int pos;
  if (is_q && p.do_q == 4) {
    // the table by position: this thread's row is a position, not a token
    t = blockIdx.x * TPP + threadIdx.x / TPV;
    if (t >= p.table_rows) return;
    pos = t;
  } else {
    if (t >= segs.start[segs.n]) return;
    int lo = 0, hi = segs.n;  // largest s with start[s] <= t
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (segs.start[mid] <= t) lo = mid; else hi = mid;
    }
    pos = segs.pos0[lo] + (t - segs.start[lo]);
  }
  const int grp = is_q ? blockIdx.y : blockIdx.y - groups_q;
  const int n_heads = is_q ? p.n_q_heads : p.n_kv_heads;
  const int h_begin = grp * p.heads_per_thread;
  const int h_end = min(n_heads, h_begin + p.heads_per_thread);
  const uint16_t *src = (is_q ? p.q_src : p.k_src) + (int64_t)t * (is_q ? p.q_st : p.k_st) + c * VEC;
  uint16_t *dst = (is_q ? p.q_dst : p.k_dst) + (int64_t)t * (is_q ? p.qd_st : p.kd_st) + c * VEC;
  const int64_t src_sh = is_q ? p.q_sh : p.k_sh, dst_sh = is_q ? p.qd_sh : p.kd_sh;
  const float scale = is_q ? p.q_scale : 1.0f;

  float cs[VEC], sn[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    int j;
    if (LAYOUT == 0)  // interleaved: pairs live inside each chunk
      j = (e < VEC / 2) ? c * (VEC / 2) + e : (c + CH / 2) * (VEC / 2) + (e - VEC / 2);
    else  // half: element e of chunk c pairs with element e of chunk c + CH/2
      j = c * VEC + e;
    sincos_phase(rope_phase(pos, rt.turns[j]), cs[e], sn[e]);
    if (scale != 1.0f) {
      cs[e] *= scale;
      sn[e] *= scale;
    }
  }
  if (is_q && (p.do_q == 2 || p.do_q == 4 || (p.do_q == 3 && grp == 0))) {
    // the factors themselves, for the attention core to rotate q with: entry j at [t][j] = (cos, sin)
    float2 *row = reinterpret_cast<float2 *>(p.q_table) + (int64_t)t * (D / 2);
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      int j;
      if (LAYOUT == 0)
        j = (e < VEC / 2) ? c * (VEC / 2) + e : (c + CH / 2) * (VEC / 2) + (e - VEC / 2);
      else
        j = c * VEC + e;
      row[j] = make_float2(cs[e], sn[e]);
    }
    if (p.do_q == 2 || p.do_q == 4) return;
  }
#pragma unroll 4
  for (int h = h_begin; h < h_end; ++h) {
    const u32x4_t xa = *reinterpret_cast<const u32x4_t *>(src + h * src_sh);
    const u32x4_t xb = *reinterpret_cast<const u32x4_t *>(src + h * src_sh + (CH / 2) * VEC);
    u32x4_t ya, yb;
    if (LAYOUT == 0) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a0 = bf16_lo(xa[e]), a1 = bf16_hi(xa[e]);
        ya[e] = pack_bf16(cs[e] * a0 - sn[e] * a1, sn[e] * a0 + cs[e] * a1);
        const float b0 = bf16_lo(xb[e]), b1 = bf16_hi(xb[e]);
        yb[e] = pack_bf16(cs[4 + e] * b0 - sn[4 + e] * b1, sn[4 + e] * b0 + cs[4 + e] * b1);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a0 = bf16_lo(xa[e]), a1 = bf16_hi(xa[e]), b0 = bf16_lo(xb[e]), b1 = bf16_hi(xb[e]);
        ya[e] = pack_bf16(cs[2 * e] * a0 - sn[2 * e] * b0, cs[2 * e + 1] * a1 - sn[2 * e + 1] * b1);
        yb[e] = pack_bf16(sn[2 * e] * a0 + cs[2 * e] * b0, sn[2 * e + 1] * a1 + cs[2 * e + 1] * b1);
      }
    }
    *reinterpret_cast<u32x4_t *>(dst + h * dst_sh) = ya;
    *reinterpret_cast<u32x4_t *>(dst + h * dst_sh + (CH / 2) * VEC) = yb;
  }
}

// rots: a small table of rotations to fill in the same launch, or null
template <int D, typename Segs>
hipError_t launch_d(RopePrepassParams p, const Segs &segs, const RopeTable &rt, const RopeRotsSmall *rots,
                    hipStream_t stream) {
  constexpr int TPP = kThreads / (D / 8 / 2);
  const int64_t tokens = (int64_t)segs.start[segs.n] - segs.start[0];
  const int groups = q_groups(p) + (p.do_k ? (p.n_kv_heads + p.heads_per_thread - 1) / p.heads_per_thread : 0);
  if (tokens <= 0 || groups == 0) return hipSuccess;
  // (a table by position has rows of its own to cover; it never has more of them than the call has tokens)
  const int64_t span = std::max<int64_t>(tokens, p.do_q == 4 ? p.table_rows : 0);
  const unsigned gx = (unsigned)((span + TPP - 1) / TPP);
  RopeRotsSmall none;
  unsigned rot_rows = 0;
  if (rots) {
    const int64_t entries = (int64_t)p.n_rot * (D / 2);
    rot_rows = (unsigned)((entries + (int64_t)gx * kThreads - 1) / ((int64_t)gx * kThreads));
  } else {
    p.n_rot = 0;
    memset(&none, 0, sizeof(none));
  }
  dim3 grid(gx, (unsigned)groups + rot_rows, 1);
  if (p.layout == 0)
    hipLaunchKernelGGL((rope_prepass_kernel<D, 0, Segs>), grid, dim3(kThreads), 0, stream, p, segs, rt, rots ? *rots : none);
  else
    hipLaunchKernelGGL((rope_prepass_kernel<D, 1, Segs>), grid, dim3(kThreads), 0, stream, p, segs, rt, rots ? *rots : none);
  return hipGetLastError();
}

template <typename Segs>
hipError_t launch_rope_prepass_t(const RopePrepassParams &p, const Segs &segs, const RopeRots *rots,
                                 const RopeRotsSmall *rots_small, const RopeTable &rt, hipStream_t stream) {
  // a large table of rotations gets a launch of its own; a small one rides along with the rows
  const bool want_rot = p.rot_dst && p.n_rot > 0;
  if (want_rot && rots) {
    const int entries = p.n_rot * (p.head_dim / 2);
    hipLaunchKernelGGL((rope_rot_table_kernel<kBlkMaxBlocks>), dim3((entries + kThreads - 1) / kThreads),
                       dim3(kThreads), 0, stream, p.rot_dst, p.n_rot, p.head_dim / 2, *rots, rt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const RopeRotsSmall *ride = (want_rot && !rots) ? rots_small : nullptr;
  if (p.head_dim == 128) return launch_d<128>(p, segs, rt, ride, stream);
  if (p.head_dim == 64) return launch_d<64>(p, segs, rt, ride, stream);
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_rope_prepass(const RopePrepassParams &p, const RopeSegs &segs, const RopeRots *rots,
                               const RopeRotsSmall *rots_small, const RopeTable &rt, hipStream_t stream) {
  return launch_rope_prepass_t(p, segs, rots, rots_small, rt, stream);
}
hipError_t launch_rope_prepass(const RopePrepassParams &p, const RopeSegsSmall &segs, const RopeRots *rots,
                               const RopeRotsSmall *rots_small, const RopeTable &rt, hipStream_t stream) {
  return launch_rope_prepass_t(p, segs, rots, rots_small, rt, stream);
}

}  // namespace ba
