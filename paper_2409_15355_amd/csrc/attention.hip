// Block-attention core for gfx950 (arXiv 2409.15355, Section 2.1 and Section 2.5).
//
// One kernel serves both attention steps.  A "problem" is a run of query tokens that
// attends (a) to a fully visible context segment and (b) causally to its own tokens:
//   - per-block encoding (Section 2.1):   no context, one problem per passage block;
//   - final block (Section 2.5):          context = concatenated cached KV, one problem
//                                         per prompt.
// Blocks never see each other because each problem only ever walks its own key range:
// masked tiles of the block-diagonal mask are never issued.
//
// Mapping onto the hardware
//   - A workgroup (8 wavefronts, two per SIMD) owns 256 packed query rows of one KV head;
//     each wave owns 32 of them.  Row r = token * G + head_in_group packs the G query heads
//     of a GQA group next to each other, so one K/V tile streamed through LDS serves all.
//   - K/V tiles (64 keys) go from HBM straight into LDS with LDS-direct loads
//     (global_load_lds_dwordx4), several tiles ahead of their use, one barrier per tile.
//   - Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: keys
//     run along accumulator registers and queries along lanes, so row reductions stay in
//     registers plus one half-wave exchange, and the exponentials are already in the
//     B-operand layout of the second contraction O^T = V^T P^T.
//   - V^T fragments come straight out of the row-major V tile with the LDS transpose
//     read (ds_read_b64_tr_b16); K fragments with 16-byte reads.  Both tiles use an XOR
//     swizzle so that neither the tile fill nor the fragment reads conflict.
//   - Softmax in fp32, log2 domain.  Q is pre-multiplied by scale * log2(e) and the score
//     accumulators START at minus the row's reference, so the MFMA result is directly the
//     exponent; the reference is set by the first tile and moved only if an exponential
//     threatens to overflow (any reference gives the same quotient sum(p v) / sum(p)).
//     P is rounded to bf16 for the second MFMA; row sums stay in fp32; the output is rounded once.
//   - The two waves of a SIMD run half an iteration apart ("ping-pong"): while one is in its
//     exponentials (VALU), the other is in an MFMA phase.
//   - The KV range can be cut into n_splits pieces; each piece writes un-normalised
//     fp32 partials (reference, sum, O) that combine_kernel merges in a fixed order.
#include <type_traits>

#include "ba_device.h"

namespace ba {
namespace {

constexpr int kCombineThreads = 256;
constexpr int kWaves = kTileRows / 32;  // 8: each wave owns one 32-query MFMA column group
constexpr int kThreads = kWaves * 64;
constexpr int kXcds = 8;        // MI355X: workgroup ids go round-robin over 8 XCDs
constexpr int kNumKBuf = 4;     // K tiles resident in LDS (role B reads one tile ahead)
constexpr int kNumVBuf = 3;     // V tiles resident in LDS
constexpr float kRebaseAbove = 1099511627776.0f;  // 2^40: a tile sum beyond this moves the reference

template <int D>
struct Geo {
  static constexpr int KCH = D / 16;          // k-steps of the QK contraction
  static constexpr int DT = D / 32;           // 32-row slabs of O^T
  static constexpr int CPR = D / 8;           // 16-byte chunks per K/V row
  static constexpr int ROWB = D * 2;          // bytes per K/V row in LDS
  static constexpr int LPR = 256 / ROWB;      // rows per 256-byte LDS line (1 or 2)
  static constexpr int GPR = ROWB / 64;       // 64-byte granules per row
  static constexpr int TILEB = kTileKeys * ROWB;
  static constexpr int RPI = 1024 / ROWB;     // rows filled by one LDS-direct wave instruction
  static constexpr int IPW = kTileKeys / RPI / (kWaves / 2);  // such instructions per COPYING wave per tile
  static constexpr size_t LDS = (size_t)(kNumKBuf + kNumVBuf) * TILEB;
};

struct Problem {
  int q_tok0;   // first query token (row of q / o / kf / vf)
  int lq;       // query tokens
  int ctx0;     // first context row
  int tctx;     // context rows
  int qpos0;    // position of query token 0
  int jt;       // row tile inside the problem
};

__device__ __forceinline__ int find_segment(const int32_t *tile_start, int n, int tile) {
  int lo = 0, hi = n;  // largest i with tile_start[i] <= tile
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (tile_start[mid] <= tile) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ Problem locate(const EncodeMeta &m, int tile) {
  int b = find_segment(m.tile_start, m.n, tile);
  Problem pr;
  pr.q_tok0 = m.offs[b];
  pr.lq = m.offs[b + 1] - m.offs[b];
  pr.ctx0 = 0;
  pr.tctx = 0;
  pr.qpos0 = 0;
  pr.jt = tile - m.tile_start[b];
  return pr;
}
__device__ __forceinline__ Problem locate(const FinalMeta &m, int tile) {
  int n = find_segment(m.tile_start, m.n, tile);
  Problem pr;
  pr.q_tok0 = m.cu_q[n];
  pr.lq = m.cu_q[n + 1] - m.cu_q[n];
  pr.ctx0 = m.cu_ctx[n];
  pr.tctx = m.cu_ctx[n + 1] - m.cu_ctx[n];
  pr.qpos0 = m.pos0[n];
  pr.jt = tile - m.tile_start[n];
  return pr;
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
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(offset), "s"(base), "s"(lds_base)
               : "memory");
}
// Wait until at most NEWER of this wave's vector-memory operations are still in flight
// (they complete in order), leaving the other counters alone.  gfx9 encoding of s_waitcnt.
template <int NEWER>
__device__ __forceinline__ void dma_wait() {
  static_assert(NEWER >= 0 && NEWER < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0f70 | (NEWER & 15) | ((NEWER >> 4) << 14));
  asm volatile("" ::: "memory");
}

#ifdef BA_TRACE
// Debug build only: per-phase timestamps of one workgroup, read back by ba_debug_read_trace().
constexpr int kTraceTiles = 80, kTraceMarks = 8;
__device__ long long g_trace[8][kTraceTiles][kTraceMarks];
#define BA_MARK(tile, m)                                                                   \
  do {                                                                                     \
    if (trace_on && (tile) < kTraceTiles && lane == 0) g_trace[wave][tile][m] = clock64(); \
  } while (0)
#else
#define BA_MARK(tile, m) do { } while (0)
#endif

template <int D, typename Meta>
__global__ __launch_bounds__(kThreads) void attn_kernel(AttnParams p, Meta meta, RopeTable rt) {
  using G = Geo<D>;
  constexpr bool kFinal = std::is_same<Meta, FinalMeta>::value;
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char *smem = (lds_char *)smem_generic;
  // LDS map: kNumKBuf K buffers from byte 0, then kNumVBuf V buffers, TILEB bytes each.
  constexpr uint32_t TB = G::TILEB;
  constexpr uint32_t VBASE = kNumKBuf * TB;

  // ---- which work item -------------------------------------------------------------------
  int id = blockIdx.x;
  if (kFinal) {
    // Consecutive work items share K/V tiles (same KV head and split, different row tile);
    // the dispatcher deals workgroup ids round-robin to the XCDs, so regroup ids such that
    // each XCD (and its L2) gets a contiguous run of work items.
    const int n_wg = gridDim.x, q = n_wg / kXcds, r = n_wg % kXcds, x = id % kXcds;
    id = x * q + min(x, r) + id / kXcds;
  }
  const int rowtile = kFinal ? id % p.total_tiles : p.total_tiles - 1 - id % p.total_tiles;
  id /= p.total_tiles;
  const int kvh = id % p.n_kv_heads;
  const int split = id / p.n_kv_heads;
  const Problem pr = locate(meta, rowtile);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform, lives in an SGPR
  const int col = lane & 31;  // query column inside the 32-wide MFMA group
  const int hf = lane >> 5;   // which half of the wave
#ifdef BA_TRACE
  const bool trace_on = blockIdx.x == 17;
#endif
  BA_MARK(79, 0);
  const int Gq = p.group;
  const int n_rows = pr.lq * Gq;
  const int row0 = pr.jt * kTileRows;

  // ---- key tiles this work item walks ---------------------------------------------------
  const int n_ctx_tiles = (pr.tctx + kTileKeys - 1) / kTileKeys;
  const int last_row = min(n_rows, row0 + kTileRows) - 1;
  const int last_tok = last_row / Gq;
  const int n_causal_tiles = last_tok / kTileKeys + 1;
  const int nt = n_ctx_tiles + n_causal_tiles;
  const int t_begin = (int)((int64_t)nt * split / p.n_splits);
  const int t_end = (int)((int64_t)nt * (split + 1) / p.n_splits);
  const int n_t = t_end - t_begin;

  // ---- Q fragments (B operand of S^T = K Q^T): rotated in registers if asked, and multiplied
  //      by scale * log2(e) before the one rounding to bf16 -----------------------------------------
  const float c2 = p.scale_log2e;
  bf16x8_t qf[G::KCH];
  const int my_row = row0 + wave * 32 + col;
  const bool row_ok = my_row < n_rows;
  const int my_tok = my_row / Gq;  // query token (inside the problem) of this lane's column
  {
    const int g = my_row - my_tok * Gq;
    const int head = kvh * Gq + g;
    const uint16_t *qp = p.q + (int64_t)(pr.q_tok0 + my_tok) * p.q_st + (int64_t)head * p.q_sh + hf * 8;
    u32x4_t raw[G::KCH];
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) {
      u32x4_t z = {0u, 0u, 0u, 0u};
      raw[kk] = row_ok ? *reinterpret_cast<const u32x4_t *>(qp + kk * 16) : z;
    }
    if (p.rope_q) {
      const int pos = pr.qpos0 + my_tok;
      if (p.rope_layout == 0) {
#pragma unroll
        for (int kk = 0; kk < G::KCH; ++kk) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float c, s;
            sincos_phase(rope_phase(pos, rt.turns[kk * 8 + hf * 4 + e]), c, s);
            c *= c2;
            s *= c2;
            float x = bf16_lo(raw[kk][e]), y = bf16_hi(raw[kk][e]);
            raw[kk][e] = pack_bf16(c * x - s * y, s * x + c * y);
          }
        }
      } else {
#pragma unroll
        for (int kk = 0; kk < G::KCH / 2; ++kk) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float c0, s0, c1, s1;
            const int j = kk * 16 + hf * 8 + 2 * e;
            sincos_phase(rope_phase(pos, rt.turns[j]), c0, s0);
            sincos_phase(rope_phase(pos, rt.turns[j + 1]), c1, s1);
            c0 *= c2; s0 *= c2; c1 *= c2; s1 *= c2;
            uint32_t wa = raw[kk][e], wb = raw[kk + G::KCH / 2][e];
            float xa0 = bf16_lo(wa), xa1 = bf16_hi(wa), xb0 = bf16_lo(wb), xb1 = bf16_hi(wb);
            raw[kk][e] = pack_bf16(c0 * xa0 - s0 * xb0, c1 * xa1 - s1 * xb1);
            raw[kk + G::KCH / 2][e] = pack_bf16(s0 * xa0 + c0 * xb0, s1 * xa1 + c1 * xb1);
          }
        }
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          raw[kk][e] = pack_bf16(bf16_lo(raw[kk][e]) * c2, bf16_hi(raw[kk][e]) * c2);
    }
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) qf[kk] = __builtin_bit_cast(bf16x8_t, raw[kk]);
  }
  BA_MARK(79, 1);

  // ---- per-lane LDS read offsets, relative to a tile buffer; the rest of an address is a
  //      wave-uniform buffer offset plus compile-time constants ------------------------------------
  uint32_t k_rd[G::KCH];  // K fragment (keys 0..31): row `col`, chunk 2 kk + hf, swizzled
  {
    const int swz = (col / G::LPR) & (G::CPR - 1);
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) k_rd[kk] = col * G::ROWB + (((kk * 2 + hf) ^ swz) << 4);
  }
  uint32_t v_rd[G::DT];  // V^T fragment (16-key step 0, low half)
  {
    const int vrow = hf * 4 + ((lane & 15) >> 2);
    const int vwithin = ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
    const int swz = (vrow / G::LPR) & (G::GPR - 1);
#pragma unroll
    for (int dt = 0; dt < G::DT; ++dt) v_rd[dt] = vrow * G::ROWB + ((dt ^ swz) << 6) + vwithin;
  }

  // ---- tile fill: which source chunk each lane fetches for its fixed LDS position ----------------
  // One wave instruction fills 1024 contiguous LDS bytes, lane i writing [16 i, 16 i + 16); the
  // swizzle is applied on the GLOBAL side.  Rows at or beyond a tile's valid count re-read its
  // last valid row: their scores are masked, and a finite duplicate keeps 0 * v equal to 0.
  const char *kc_base = (const char *)(p.kc + (int64_t)pr.ctx0 * p.kc_st + (int64_t)kvh * p.kc_sh);
  const char *vc_base = (const char *)(p.vc + (int64_t)pr.ctx0 * p.vc_st + (int64_t)kvh * p.vc_sh);
  const char *kf_base = (const char *)(p.kf + (int64_t)pr.q_tok0 * p.kf_st + (int64_t)kvh * p.kf_sh);
  const char *vf_base = (const char *)(p.vf + (int64_t)pr.q_tok0 * p.vf_st + (int64_t)kvh * p.vf_sh);
  const uint32_t kc_rb = (uint32_t)p.kc_st * 2u, vc_rb = (uint32_t)p.vc_st * 2u;  // row strides, bytes
  const uint32_t kf_rb = (uint32_t)p.kf_st * 2u, vf_rb = (uint32_t)p.vf_st * 2u;
  const bool prim_ctx = n_ctx_tiles > 0;  // the segment whose full tiles get cached lane offsets
  int g_row[G::IPW];
  uint32_t g_kchunk[G::IPW], g_vchunk[G::IPW];  // byte offset of the source chunk inside its row
  uint32_t k_src[G::IPW], v_src[G::IPW];        // full per-lane byte offsets for a full primary tile
#pragma unroll
  for (int i = 0; i < G::IPW; ++i) {
    const int row = ((wave & (kWaves / 2 - 1)) * G::IPW + i) * G::RPI + lane / G::CPR;
    const int pos = lane % G::CPR;
    g_row[i] = row;
    g_kchunk[i] = (uint32_t)(pos ^ ((row / G::LPR) & (G::CPR - 1))) << 4;
    g_vchunk[i] = (uint32_t)((((pos >> 2) ^ ((row / G::LPR) & (G::GPR - 1))) << 2) | (pos & 3)) << 4;
    k_src[i] = (uint32_t)row * (prim_ctx ? kc_rb : kf_rb) + g_kchunk[i];
    v_src[i] = (uint32_t)row * (prim_ctx ? vc_rb : vf_rb) + g_vchunk[i];
  }
  // (only waves 0..3 copy: they have slack at the end of every iteration, see below)
  const uint32_t lds_wave = (uint32_t)(uintptr_t)smem + (wave & (kWaves / 2 - 1)) * G::IPW * 1024;
  auto issue_k = [&](int t, uint32_t dst) {  // tile t of the problem -> LDS byte offset dst
    const bool isctx = t < n_ctx_tiles;
    const int tc = isctx ? t : t - n_ctx_tiles;
    const uint32_t rb = isctx ? kc_rb : kf_rb;
    const char *ptr = (isctx ? kc_base : kf_base) + (uint64_t)(uint32_t)tc * (uint64_t)(rb * (uint32_t)kTileKeys);
    const int valid = min(kTileKeys, (isctx ? pr.tctx : pr.lq) - tc * kTileKeys);
    if (valid == kTileKeys && isctx == prim_ctx) {
#pragma unroll
      for (int i = 0; i < G::IPW; ++i) lds_dma16(ptr, k_src[i], lds_wave + dst + i * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < G::IPW; ++i)
        lds_dma16(ptr, (uint32_t)min(g_row[i], valid - 1) * rb + g_kchunk[i], lds_wave + dst + i * 1024);
    }
  };
  auto issue_v = [&](int t, uint32_t dst) {
    const bool isctx = t < n_ctx_tiles;
    const int tc = isctx ? t : t - n_ctx_tiles;
    const uint32_t rb = isctx ? vc_rb : vf_rb;
    const char *ptr = (isctx ? vc_base : vf_base) + (uint64_t)(uint32_t)tc * (uint64_t)(rb * (uint32_t)kTileKeys);
    const int valid = min(kTileKeys, (isctx ? pr.tctx : pr.lq) - tc * kTileKeys);
    if (valid == kTileKeys && isctx == prim_ctx) {
#pragma unroll
      for (int i = 0; i < G::IPW; ++i) lds_dma16(ptr, v_src[i], lds_wave + dst + i * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < G::IPW; ++i)
        lds_dma16(ptr, (uint32_t)min(g_row[i], valid - 1) * rb + g_vchunk[i], lds_wave + dst + i * 1024);
    }
  };

  // ---- running state -----------------------------------------------------------------------------
  f32x16_t oacc[G::DT];
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
  float mb = 0.f;      // the row's reference, log2 units
  f32x16_t negmb;      // -mb in every entry: where the score accumulators start
#pragma unroll
  for (int v = 0; v < 16; ++v) negmb[v] = 0.f;
  float l_run = 0.f;   // this lane's share of the running sum of exponentials
  const int first_tok_wave = (row0 + wave * 32) / Gq;

  // S'^T = K Q'^T - reference, from the K tile at LDS byte offset kofs: sacc[a] is keys
  // 32a..32a+31 x this wave's 32 queries, already the base-2 exponent.  The 2 * KCH steps go in
  // groups of four; a group's K fragments are read while the previous group's MFMAs run.
  auto qk = [&](uint32_t kofs, f32x16_t (&sacc)[2]) {
    constexpr int STEPS = 2 * G::KCH;  // step = kk * 2 + a: consecutive MFMAs are independent
    constexpr int GS = 4;
    constexpr int NG = STEPS / GS;
    auto read_k = [&](int step) {
      const int a = step & 1, kk = step >> 1;
      return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(
          smem + (k_rd[kk] + kofs) + a * 32 * G::ROWB);
    };
    bf16x8_t fr[2][GS];
#pragma unroll
    for (int j = 0; j < GS; ++j) fr[0][j] = read_k(j);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      if (g + 1 < NG) {
#pragma unroll
        for (int j = 0; j < GS; ++j) fr[(g + 1) & 1][j] = read_k((g + 1) * GS + j);
      }
#pragma unroll
      for (int j = 0; j < GS; ++j) {
        const int step = g * GS + j, a = step & 1, kk = step >> 1;
        sacc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][j], qf[kk], kk == 0 ? negmb : sacc[a], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Row maxima of a score tile, then move the reference there: exponents, running sum and
  // output accumulators are all re-expressed relative to the new reference.  Runs on a wave's
  // first tile and, after that, only when an exponential grew past kRebaseAbove.
  auto rebase = [&](f32x16_t (&sacc)[2], bool first) {
    float m0 = sacc[0][0];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) m0 = fmaxf(m0, sacc[a][v]);
    const float mx = fmaxf(m0, other_half(m0));
    // first tile: take the maximum whatever its sign (nothing visible: keep 0); later: only raise
    const float shift = first ? (mx == -INFINITY ? 0.f : mx) : fmaxf(mx, 0.f);
    const float alpha = first ? 1.f : __builtin_amdgcn_exp2f(-shift);
    mb += shift;
#pragma unroll
    for (int v = 0; v < 16; ++v) negmb[v] = -mb;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[a][v] -= shift;
    l_run *= alpha;
#pragma unroll
    for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
  };
  // P = 2^S' rounded to bf16 (the B operand of PV); returns this lane's fp32 sum of the exponentials
  auto exponentials = [&](const f32x16_t (&sacc)[2], bf16x8_t (&pf)[4]) {
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        u32x4_t w;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float p0 = __builtin_amdgcn_exp2f(sacc[a][e * 8 + 2 * i]);
          const float p1 = __builtin_amdgcn_exp2f(sacc[a][e * 8 + 2 * i + 1]);
          s0 += p0;
          s1 += p1;
          w[i] = pack_bf16(p0, p1);
        }
        pf[a * 2 + e] = __builtin_bit_cast(bf16x8_t, w);
      }
    }
    return s0 + s1;
  };
  // The softmax step of one tile: mask where needed (diagonal and ragged tiles only), turn the
  // exponents into P, and keep the running sum.  All branches are wave-uniform.
  auto softmax = [&](int t, bool first, f32x16_t (&sacc)[2], bf16x8_t (&pf)[4]) {
    const bool isctx = t < n_ctx_tiles;
    const int tc = isctx ? t : t - n_ctx_tiles;
    const int valid = min(kTileKeys, (isctx ? pr.tctx : pr.lq) - tc * kTileKeys);
    const int key0 = tc * kTileKeys;
    const bool need_mask = isctx ? (valid < kTileKeys) : (key0 + kTileKeys - 1 > first_tok_wave) || (valid < kTileKeys);
    if (need_mask) {
      asm volatile("" ::: "memory");  // keep this a real branch: never speculate the selects
      const int lim = isctx ? valid : min(my_tok - key0 + 1, valid);  // visible keys in this tile
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = a * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
          if (key >= lim) sacc[a][v] = -INFINITY;
        }
    }
    if (first) {
      asm volatile("" ::: "memory");
      rebase(sacc, true);
    }
    float tsum = exponentials(sacc, pf);
    if (__builtin_amdgcn_ballot_w64(!(tsum < kRebaseAbove)) != 0) {  // overflow guard: practically never
      asm volatile("" ::: "memory");
      rebase(sacc, false);
      tsum = exponentials(sacc, pf);
    }
    l_run += tsum;
  };
  // O^T += V^T P^T from the V tile at LDS byte offset vofs; fragments of a 16-key step are
  // read one step ahead of the MFMAs that consume them.
  auto pv_mma = [&](uint32_t vofs, const bf16x8_t (&pf)[4]) {
    typedef __attribute__((address_space(3))) s16x4_t lds_s16x4;
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    auto read_v = [&](int kc, int dt) {
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4 *)(smem + (v_rd[dt] + vofs) + kc * 16 * G::ROWB));
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4 *)(smem + (v_rd[dt] + vofs) + (kc * 16 + 8) * G::ROWB));
      const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8_t, both);
    };
    bf16x8_t fr[2][G::DT];
#pragma unroll
    for (int dt = 0; dt < G::DT; ++dt) fr[0][dt] = read_v(0, dt);
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) {
      if (kc + 1 < 4) {
#pragma unroll
        for (int dt = 0; dt < G::DT; ++dt) fr[(kc + 1) & 1][dt] = read_v(kc + 1, dt);
      }
#pragma unroll
      for (int dt = 0; dt < G::DT; ++dt)
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[kc & 1][dt], pf[kc], oacc[dt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- the walk over the key tiles ------------------------------------------------------------------
  // Tile i (counted from t_begin) has its K in K buffer i % 4 and its V in V buffer i % 3.  At the
  // start of iteration i the copying waves start the copies of K(i+3) and V(i+2); at its end they wait
  // for the copies started one iteration EARLIER (K(i+2), V(i+1)), then all waves meet at the
  // barrier.  Waves 0..3 (role A) run  QK(i), softmax(i), PV(i)  inside iteration i; waves 4..7
  // (role B) run  softmax(i), PV(i), QK(i+1).  Waves w and w + 4 share a SIMD, so while one is
  // in its VALU phase the other is in an MFMA phase instead of both queueing for the same unit.
  // Role B is the longer chain (the SIMD arbitrates oldest wave first), so role A alone issues
  // the copies and waits for them.
  const bool role_b = wave >= kWaves / 2;
  uint32_t vo0 = VBASE, vo1 = VBASE + TB, vo2 = VBASE + 2 * TB;  // V buffers of tiles i, i+1, i+2
  if (!role_b && n_t > 0) {
    issue_k(t_begin, 0);
    issue_v(t_begin, vo0);
    if (n_t > 1) {
      issue_k(t_begin + 1, TB);
      issue_v(t_begin + 1, vo1);
    }
    if (n_t > 2) issue_k(t_begin + 2, 2 * TB);
  }
  BA_MARK(79, 2);
  dma_wait<0>();  // unconditional: the Q fragment loads are then known to be complete in the loops
  __syncthreads();
  BA_MARK(79, 3);
  // one iteration's copies (role A only) and the end of an iteration
  auto start_copies = [&](int i) {
    if (i + 3 < n_t) issue_k(t_begin + i + 3, ((i + 3) & (kNumKBuf - 1)) * TB);
    if (i + 2 < n_t) issue_v(t_begin + i + 2, vo2);
  };
  auto rotate_v = [&]() {
    const uint32_t v_t = vo0;
    vo0 = vo1;
    vo1 = vo2;
    vo2 = v_t;
  };
  if (!role_b) {
#pragma unroll 1
    for (int i = 0; i < n_t; ++i) {
      start_copies(i);
      f32x16_t sacc[2];
      bf16x8_t pf[4];
      BA_MARK(i, 0);
      qk((i & (kNumKBuf - 1)) * TB, sacc);
      BA_MARK(i, 1);
      softmax(t_begin + i, i == 0, sacc, pf);
      BA_MARK(i, 2);
      pv_mma(vo0, pf);
      BA_MARK(i, 3);
      rotate_v();
      if (i + 3 < n_t) dma_wait<2 * G::IPW>(); else dma_wait<0>();
      BA_MARK(i, 4);
      __syncthreads();  // K(i+2) and V(i+1) have landed; the buffers of tile i are free
      BA_MARK(i, 5);
    }
  } else {
    f32x16_t sacc[2];
    if (n_t > 0) qk(0, sacc);
#pragma unroll 1
    for (int i = 0; i < n_t; ++i) {
      bf16x8_t pf[4];
      BA_MARK(i, 0);
      softmax(t_begin + i, i == 0, sacc, pf);
      BA_MARK(i, 1);
      pv_mma(vo0, pf);
      BA_MARK(i, 2);
      if (i + 1 < n_t) qk(((i + 1) & (kNumKBuf - 1)) * TB, sacc);
      BA_MARK(i, 3);
      rotate_v();
      BA_MARK(i, 4);
      __syncthreads();
      BA_MARK(i, 5);
    }
  }
  BA_MARK(79, 4);
  static_assert((kNumKBuf & (kNumKBuf - 1)) == 0 && kNumVBuf == 3, "buffer rotation above assumes 4 and 3");

  // ---- epilogue: each wave transposes its O^T through its own slice of LDS, half of the head
  //      dimension at a time, so that rows leave as contiguous lines (all waves are past the
  //      loop's last barrier, and nothing else touches LDS any more) ---------------------------------
  constexpr int HD = D / 2;               // floats per staged row piece
  constexpr int HCH = HD / 4;             // 16-byte chunks per piece (16 or 8)
  constexpr int PITCH = HD * 4;           // bytes per staged row piece (256 or 128)
  constexpr int HLPR = 256 / PITCH;       // pieces per 256-byte LDS line
  lds_char *stage = smem + wave * (32 * PITCH);
  const float l_tot = l_run + other_half(l_run);
  const float inv = (p.n_splits == 1) ? 1.0f / l_tot : 1.0f;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    // write: lane (col, hf) owns query row `col`; chunk index XOR row keeps banks apart
#pragma unroll
    for (int dh = 0; dh < G::DT / 2; ++dh) {
      const int dt = half * (G::DT / 2) + dh;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int chunk = dh * 8 + q4 * 2 + hf;  // 16-byte chunk inside the piece
        f32x4_t w = {oacc[dt][q4 * 4 + 0] * inv, oacc[dt][q4 * 4 + 1] * inv, oacc[dt][q4 * 4 + 2] * inv,
                     oacc[dt][q4 * 4 + 3] * inv};
        *reinterpret_cast<__attribute__((address_space(3))) f32x4_t *>(
            stage + col * PITCH + ((chunk ^ ((col / HLPR) & (HCH - 1))) << 4)) = w;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // read back row-major: HCH lanes per row piece, 64 / HCH rows per pass
    constexpr int ROWS_PP = 64 / HCH;
#pragma unroll
    for (int pass = 0; pass < 32 / ROWS_PP; ++pass) {
      const int rr = pass * ROWS_PP + lane / HCH;  // row inside this wave's 32
      const int ch = lane % HCH;
      const f32x4_t w = *reinterpret_cast<const __attribute__((address_space(3))) f32x4_t *>(
          stage + rr * PITCH + ((ch ^ ((rr / HLPR) & (HCH - 1))) << 4));
      const int r = row0 + wave * 32 + rr;
      if (r < n_rows) {
        const int i = r / Gq;
        const int g = r - i * Gq;
        const int head = kvh * Gq + g;
        const int d = half * HD + ch * 4;
        if (p.n_splits == 1) {
          uint2 o2;
          o2.x = pack_bf16(w[0], w[1]);
          o2.y = pack_bf16(w[2], w[3]);
          *reinterpret_cast<uint2 *>(p.o + (int64_t)(pr.q_tok0 + i) * p.o_st + (int64_t)head * p.o_sh + d) = o2;
        } else {
          const int64_t prow = (int64_t)(pr.q_tok0 + i) * p.n_q_heads + head;
          *reinterpret_cast<f32x4_t *>(p.part_o + ((int64_t)split * p.part_rows + prow) * D + d) = w;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if (p.n_splits > 1 && hf == 0 && row_ok) {
    const int g = my_row - my_tok * Gq;
    const int64_t prow = (int64_t)(pr.q_tok0 + my_tok) * p.n_q_heads + kvh * Gq + g;
    float2 ml = {l_tot > 0.f ? mb : -INFINITY, l_tot};  // reference in log2 units; -inf: nothing visible
    *reinterpret_cast<float2 *>(p.part_ml + ((int64_t)split * p.part_rows + prow) * 2) = ml;
  }
  BA_MARK(79, 5);
}

// Merge split partials in split order: m = max m_i, w_i = 2^(m_i - m),
// o = sum_i w_i O_i / sum_i w_i l_i.
template <int D>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(AttnParams p, int64_t n_rows) {
  constexpr int TPR = D / 4;                  // threads per row
  constexpr int RPB = kCombineThreads / TPR;  // rows per workgroup
  const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / TPR;
  if (row >= n_rows) return;
  const int d = (threadIdx.x % TPR) * 4;
  // all loads are unconditional and independent, so they go out together; a split that saw no
  // visible key wrote O = 0, l = 0 and a reference of -inf, and gets weight 0
  constexpr int MAXS = 32;  // the host never asks for more splits
  float wgt[MAXS];
  float m = -INFINITY;
#pragma unroll 8
  for (int s = 0; s < p.n_splits; ++s) {
    wgt[s & (MAXS - 1)] = p.part_ml[((int64_t)s * p.part_rows + row) * 2];
    m = fmaxf(m, wgt[s & (MAXS - 1)]);
  }
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
#pragma unroll 8
  for (int s = 0; s < p.n_splits; ++s) {
    const float ms = wgt[s & (MAXS - 1)];
    const float w = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - m);
    const float ls = p.part_ml[((int64_t)s * p.part_rows + row) * 2 + 1];
    const f32x4_t o = *reinterpret_cast<const f32x4_t *>(p.part_o + ((int64_t)s * p.part_rows + row) * D + d);
    l += w * ls;
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] += w * o[i];
  }
  const float inv = 1.0f / l;
  const int64_t tokn = row / p.n_q_heads;
  const int head = (int)(row - tokn * p.n_q_heads);
  uint2 w;
  w.x = pack_bf16(acc[0] * inv, acc[1] * inv);
  w.y = pack_bf16(acc[2] * inv, acc[3] * inv);
  *reinterpret_cast<uint2 *>(p.o + tokn * p.o_st + (int64_t)head * p.o_sh + d) = w;
}

template <int D, typename Meta>
hipError_t launch_attn_t(const AttnParams &p, const Meta &meta, const RopeTable &rt, hipStream_t stream) {
  const int64_t n_wg = (int64_t)p.total_tiles * p.n_kv_heads * p.n_splits;
  if (n_wg == 0) return hipSuccess;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  constexpr size_t lds = Geo<D>::LDS;
  static_assert((size_t)kWaves * 32 * D * 2 <= lds, "epilogue staging must fit the tile buffers");
  static_assert(lds <= 160 * 1024, "gfx950 has 160 KB of LDS per workgroup");
  static bool raised = false;  // more than 64 KB of dynamic LDS has to be asked for once per kernel
  if (!raised && lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_kernel<D, Meta>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    raised = true;
  }
  hipLaunchKernelGGL((attn_kernel<D, Meta>), dim3((unsigned)n_wg), dim3(kThreads), lds, stream, p, meta, rt);
  return hipGetLastError();
}

}  // namespace

#ifdef BA_TRACE
extern "C" int ba_debug_read_trace(long long *host_out) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_trace), sizeof(g_trace));
}
#endif

hipError_t launch_attn_encode(const AttnParams &p, const EncodeMeta &meta, const RopeTable &rt,
                              hipStream_t stream) {
  if (p.head_dim == 128) return launch_attn_t<128, EncodeMeta>(p, meta, rt, stream);
  if (p.head_dim == 64) return launch_attn_t<64, EncodeMeta>(p, meta, rt, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_attn_final(const AttnParams &p, const FinalMeta &meta, const RopeTable &rt,
                             hipStream_t stream) {
  if (p.head_dim == 128) return launch_attn_t<128, FinalMeta>(p, meta, rt, stream);
  if (p.head_dim == 64) return launch_attn_t<64, FinalMeta>(p, meta, rt, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_combine(const AttnParams &p, int64_t n_tokens, hipStream_t stream) {
  const int64_t n_rows = n_tokens * p.n_q_heads;
  if (n_rows == 0) return hipSuccess;
  if (p.head_dim == 128) {
    constexpr int RPB = kCombineThreads / (128 / 4);
    hipLaunchKernelGGL((combine_kernel<128>), dim3((unsigned)((n_rows + RPB - 1) / RPB)), dim3(kCombineThreads), 0,
                       stream, p, n_rows);
  } else if (p.head_dim == 64) {
    constexpr int RPB = kCombineThreads / (64 / 4);
    hipLaunchKernelGGL((combine_kernel<64>), dim3((unsigned)((n_rows + RPB - 1) / RPB)), dim3(kCombineThreads), 0,
                       stream, p, n_rows);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ba
