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
//   - A workgroup (8 wavefronts, two per SIMD) owns 256 packed query rows of one KV head.
//     Row r = token * G + head_in_group packs the G query heads of a GQA group next to
//     each other, so one K/V tile streamed through LDS serves all of them.
//   - K/V tiles (64 keys) go from HBM straight into LDS with LDS-direct loads
//     (global_load_lds_dwordx4), double buffered, one barrier per tile.
//   - Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: keys
//     run along accumulator registers and queries along lanes, so the softmax max/sum
//     reduce in registers plus a single half-wave exchange, and the exponentials are
//     already in the B-operand layout of the second contraction O^T = V^T P^T.
//   - V^T fragments come straight out of the row-major V tile with the LDS transpose
//     read (ds_read_b64_tr_b16); K fragments with 16-byte reads.  Both tiles use an XOR
//     swizzle so that neither the tile fill nor the fragment reads conflict.
//   - Softmax runs in fp32 in the log2 domain against a lazily raised reference; P is
//     rounded to bf16 for the second MFMA; the output is rounded once.
//   - The KV range can be cut into n_splits pieces; each piece writes un-normalised
//     fp32 partials (reference, sum, O) that combine_kernel merges in a fixed order.
#include <type_traits>

#include "ba_device.h"

namespace ba {
namespace {

constexpr int kCombineThreads = 256;
// A wave owns NB groups of 32 query rows.  NB = 1: 8 waves per workgroup, two per SIMD, so
// one wave's softmax (VALU) runs under the other's MFMAs; NB = 2: 4 waves, one per SIMD.
constexpr int kNB = 1;
constexpr bool kPipelined = false;  // software-pipeline QK of tile t+1 under the softmax of tile t
constexpr int kWaves = kTileRows / (32 * kNB);
constexpr int kThreads = kWaves * 64;
constexpr int kRowsPerWave = 32 * kNB;
constexpr float kLazyLog2 = 8.0f;                 // exponentials may reach 2^8 before the reference moves
constexpr int kXcds = 8;                          // MI355X: workgroup ids go round-robin over 8 XCDs

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
  static constexpr int IPW = kTileKeys / RPI / kWaves;  // such instructions per wave per tile
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
// HBM latency on every tile.  The price is that completion is ours to wait for: dma_wait()
// must come before the barrier that publishes the buffer.
__device__ __forceinline__ void lds_dma16(const char *base, uint32_t offset, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(offset), "s"(base), "s"(lds_base)
               : "memory");
}
__device__ __forceinline__ void dma_wait() {
  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0), leaving expcnt and lgkmcnt alone (gfx9 encoding)
  asm volatile("" ::: "memory");
}

template <int D, typename Meta>
__global__ __launch_bounds__(kThreads) void attn_kernel(AttnParams p, Meta meta, RopeTable rt) {
  using G = Geo<D>;
  constexpr bool kFinal = std::is_same<Meta, FinalMeta>::value;
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char *smem = (lds_char *)smem_generic;
  // LDS map: K buffers at 0 and TILEB, V buffers at 2*TILEB and 3*TILEB.

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
  const int col = lane & 31;  // query column inside a 32-wide MFMA group
  const int hf = lane >> 5;   // which half of the wave
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

  // ---- Q fragments (B operand of S^T = K Q^T), rotated in registers if asked -------------
  bf16x8_t qf[kNB][G::KCH];
  int tok[kNB];        // query token (inside the problem) of this lane's column(s)
  bool row_ok[kNB];
#pragma unroll
  for (int b = 0; b < kNB; ++b) {
    const int r = row0 + wave * kRowsPerWave + b * 32 + col;
    row_ok[b] = r < n_rows;
    const int i = r / Gq;
    const int g = r - i * Gq;
    tok[b] = i;
    const int head = kvh * Gq + g;
    const uint16_t *qp = p.q + (int64_t)(pr.q_tok0 + i) * p.q_st + (int64_t)head * p.q_sh + hf * 8;
    u32x4_t raw[G::KCH];
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) {
      u32x4_t z = {0u, 0u, 0u, 0u};
      raw[kk] = row_ok[b] ? *reinterpret_cast<const u32x4_t *>(qp + kk * 16) : z;
    }
    if (p.rope_q) {
      const int pos = pr.qpos0 + i;
      if (p.rope_layout == 0) {
#pragma unroll
        for (int kk = 0; kk < G::KCH; ++kk) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float c, s;
            sincos_phase(rope_phase(pos, rt.turns[kk * 8 + hf * 4 + e]), c, s);
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
            uint32_t wa = raw[kk][e], wb = raw[kk + G::KCH / 2][e];
            float xa0 = bf16_lo(wa), xa1 = bf16_hi(wa), xb0 = bf16_lo(wb), xb1 = bf16_hi(wb);
            raw[kk][e] = pack_bf16(c0 * xa0 - s0 * xb0, c1 * xa1 - s1 * xb1);
            raw[kk + G::KCH / 2][e] = pack_bf16(s0 * xa0 + c0 * xb0, s1 * xa1 + c1 * xb1);
          }
        }
      }
    }
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) qf[b][kk] = __builtin_bit_cast(bf16x8_t, raw[kk]);
  }

  // ---- per-lane LDS read offsets; everything else about an address is a compile-time
  //      constant that folds into the instruction's offset field ---------------------------------
  uint32_t k_rd[G::KCH];  // K fragment (a = 0, buffer 0): row `col`, chunk 2 kk + hf, swizzled
  {
    const int swz = (col / G::LPR) & (G::CPR - 1);
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) k_rd[kk] = col * G::ROWB + (((kk * 2 + hf) ^ swz) << 4);
  }
  uint32_t v_rd[G::DT];  // V^T fragment (kc = 0, low half, buffer 0)
  {
    const int vrow = hf * 4 + ((lane & 15) >> 2);
    const int vwithin = ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
    const int swz = (vrow / G::LPR) & (G::GPR - 1);
#pragma unroll
    for (int dt = 0; dt < G::DT; ++dt) v_rd[dt] = 2 * G::TILEB + vrow * G::ROWB + ((dt ^ swz) << 6) + vwithin;
  }
  // ---- per-lane pieces of the tile fill: row and (swizzled) source chunk of each LDS-direct load
  int g_row[G::IPW];
  uint32_t g_kchunk[G::IPW], g_vchunk[G::IPW];  // byte offset of the source chunk inside its row
#pragma unroll
  for (int i = 0; i < G::IPW; ++i) {
    const int row = (wave * G::IPW + i) * G::RPI + lane / G::CPR;
    const int pos = lane % G::CPR;
    g_row[i] = row;
    g_kchunk[i] = (uint32_t)(pos ^ ((row / G::LPR) & (G::CPR - 1))) << 4;
    g_vchunk[i] = (uint32_t)((((pos >> 2) ^ ((row / G::LPR) & (G::GPR - 1))) << 2) | (pos & 3)) << 4;
  }

  // ---- running softmax state and O^T accumulators ------------------------------------------
  f32x16_t oacc[G::DT][kNB];
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int b = 0; b < kNB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[dt][b][v] = 0.f;
  // Online softmax with a LAZY reference: exponentials are taken relative to m_ref, which
  // is raised only when a tile's maximum exceeds it by more than kLazyLog2 powers of two.
  // Any reference gives the same quotient sum(p v) / sum(p); keeping it fixed avoids
  // rescaling the O^T accumulators on almost every tile.
  float m_ref[kNB];  // reference, raw score units
  float mb[kNB];     // m_ref * scale_log2e (0 while nothing was seen)
  float l_run[kNB];  // this lane's share of the running sum
#pragma unroll
  for (int b = 0; b < kNB; ++b) {
    m_ref[b] = -INFINITY;
    mb[b] = 0.f;
    l_run[b] = 0.f;
  }
  const float c2 = p.scale_log2e;
  const float tau = kLazyLog2 / c2;
  const int first_tok_wave = (row0 + wave * kRowsPerWave) / Gq;

  // Tile t: base pointers (wave-uniform), row stride in bytes, valid rows, first key, causal?
  struct Tile {
    const char *kp, *vp;
    uint32_t kst, vst;
    int valid, key0;
    bool causal;
  };
  auto tile_of = [&](int t) {
    Tile tl;
    if (t < n_ctx_tiles) {
      const int64_t r0 = (int64_t)pr.ctx0 + (int64_t)t * kTileKeys;
      tl.kp = (const char *)(p.kc + r0 * p.kc_st + (int64_t)kvh * p.kc_sh);
      tl.vp = (const char *)(p.vc + r0 * p.vc_st + (int64_t)kvh * p.vc_sh);
      tl.kst = (uint32_t)p.kc_st * 2u;
      tl.vst = (uint32_t)p.vc_st * 2u;
      tl.valid = min(kTileKeys, pr.tctx - t * kTileKeys);
      tl.key0 = 0;
      tl.causal = false;
    } else {
      const int tc = t - n_ctx_tiles;
      const int64_t r0 = (int64_t)pr.q_tok0 + (int64_t)tc * kTileKeys;
      tl.kp = (const char *)(p.kf + r0 * p.kf_st + (int64_t)kvh * p.kf_sh);
      tl.vp = (const char *)(p.vf + r0 * p.vf_st + (int64_t)kvh * p.vf_sh);
      tl.kst = (uint32_t)p.kf_st * 2u;
      tl.vst = (uint32_t)p.vf_st * 2u;
      tl.valid = min(kTileKeys, pr.lq - tc * kTileKeys);
      tl.key0 = tc * kTileKeys;
      tl.causal = true;
    }
    return tl;
  };
  // Copy a K or V tile into LDS buffer `buf` with LDS-direct loads: one wave instruction
  // fills 1024 contiguous LDS bytes, lane i writing bytes [16 i, 16 i + 16); the swizzle is
  // applied on the GLOBAL side (each lane fetches the chunk that belongs at its LDS position).
  // Rows at or beyond `valid` re-read the last valid row: their scores are masked, and a
  // finite duplicate keeps 0 * v equal to 0.
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  auto issue_k = [&](const Tile &tl, int buf) {
#pragma unroll
    for (int i = 0; i < G::IPW; ++i) {
      const uint32_t row = (uint32_t)min(g_row[i], tl.valid - 1);
      lds_dma16(tl.kp, row * tl.kst + g_kchunk[i], lds0 + buf * G::TILEB + (wave * G::IPW + i) * 1024);
    }
  };
  auto issue_v = [&](const Tile &tl, int buf) {
#pragma unroll
    for (int i = 0; i < G::IPW; ++i) {
      const uint32_t row = (uint32_t)min(g_row[i], tl.valid - 1);
      lds_dma16(tl.vp, row * tl.vst + g_vchunk[i], lds0 + (2 + buf) * G::TILEB + (wave * G::IPW + i) * 1024);
    }
  };

  // S^T = K Q^T from K buffer BUF: sacc[a][b] is keys 32a..32a+31 x queries 32b..32b+31.
  // The 2 * KCH steps go in groups of four; a group's K fragments are read while the previous
  // group's MFMAs run, so LDS latency stays off the MFMA chain.  sched_barrier(0) pins it.
  auto qk = [&](auto buf_c, f32x16_t (&sacc)[2][kNB]) {
    constexpr int BUF = decltype(buf_c)::value;
    constexpr int STEPS = 2 * G::KCH;  // step = kk * 2 + a: consecutive MFMAs are independent
    constexpr int GS = 4;
    constexpr int NG = STEPS / GS;
    auto read_k = [&](int step) {
      const int a = step & 1, kk = step >> 1;
      return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(
          smem + k_rd[kk] + (BUF * G::TILEB + a * 32 * G::ROWB));
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
#pragma unroll
        for (int b = 0; b < kNB; ++b) {
          if (kk == 0) {
            f32x16_t z;
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = 0.f;
            sacc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][j], qf[b][kk], z, 0, 0, 0);
          } else {
            sacc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][j], qf[b][kk], sacc[a][b], 0, 0, 0);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Mask a fresh score tile where needed (diagonal and ragged tiles only), take its row maxima
  // and raise the lazy reference if a row outgrew it.  Both branches are wave-uniform and rare.
  auto mask_and_reference = [&](const Tile &tl, f32x16_t (&sacc)[2][kNB]) {
    const bool need_mask = tl.causal ? (tl.key0 + kTileKeys - 1 > first_tok_wave) || (tl.valid < kTileKeys)
                                     : (tl.valid < kTileKeys);
    if (need_mask) {
      asm volatile("" ::: "memory");  // keep this a real branch: never speculate the selects
#pragma unroll
      for (int b = 0; b < kNB; ++b) {
        const int lim = tl.causal ? min(tok[b] - tl.key0 + 1, tl.valid) : tl.valid;  // visible keys here
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = a * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
            if (key >= lim) sacc[a][b][v] = -INFINITY;
          }
      }
    }
    float mx[kNB];
    bool raise[kNB], any_raise = false;
#pragma unroll
    for (int b = 0; b < kNB; ++b) {
      float m0 = sacc[0][b][0];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) m0 = fmaxf(m0, sacc[a][b][v]);
      mx[b] = fmaxf(m0, other_half(m0));
      raise[b] = mx[b] > m_ref[b] + tau;
      any_raise = any_raise || raise[b];
    }
    if (__builtin_amdgcn_ballot_w64(any_raise) != 0) {  // rare after the first tile
      asm volatile("" ::: "memory");  // a real branch, so the accumulators are left alone otherwise
#pragma unroll
      for (int b = 0; b < kNB; ++b) {
        const float m_new = raise[b] ? mx[b] : m_ref[b];
        const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((m_ref[b] - m_new) * c2);
        m_ref[b] = m_new;
        mb[b] = (m_new == -INFINITY) ? 0.f : m_new * c2;
        l_run[b] *= alpha;
#pragma unroll
        for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[dt][b][v] *= alpha;
      }
    }
  };
  // P = 2^(S * scale_log2e - reference), summed in fp32, rounded to bf16 as the B operand of PV
  auto exponentials = [&](const f32x16_t (&sacc)[2][kNB], bf16x8_t (&pf)[kNB][4]) {
#pragma unroll
    for (int b = 0; b < kNB; ++b) {
      float sum = 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        float pv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          pv[v] = __builtin_amdgcn_exp2f(sacc[a][b][v] * c2 - mb[b]);
          sum += pv[v];
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          u32x4_t w;
#pragma unroll
          for (int i = 0; i < 4; ++i) w[i] = pack_bf16(pv[e * 8 + 2 * i], pv[e * 8 + 2 * i + 1]);
          pf[b][a * 2 + e] = __builtin_bit_cast(bf16x8_t, w);
        }
      }
      l_run[b] += sum;
    }
  };
  // Phase 1 of the pipelined iteration: the QK MFMAs of the NEXT tile and the exponentials of
  // the CURRENT one, written out interleaved.  The 2 * KCH MFMA steps (key half a outermost,
  // so that the first half of the new scores is complete when the first half of the old ones
  // has been consumed) go in eight groups; the K fragments of a group are read one group
  // ahead, and after every second group a quarter of the exponentials follows.
  // sched_barrier(0) pins the groups; inside a group the scheduler interleaves.
  auto qk_with_exponentials = [&](auto buf_c, f32x16_t (&sacc)[2][kNB], const f32x16_t (&scur)[2][kNB],
                                  bf16x8_t (&pf)[kNB][4]) {
    constexpr int BUF = decltype(buf_c)::value;
    constexpr int STEPS = 2 * G::KCH;   // step = a * KCH + kk
    constexpr int NG = 8;               // groups
    constexpr int GS = STEPS / NG;      // steps per group (2 or 1)
    auto read_k = [&](int step) {
      const int a = step / G::KCH, kk = step % G::KCH;
      return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(
          smem + k_rd[kk] + (BUF * G::TILEB + a * 32 * G::ROWB));
    };
    float sum[kNB];
#pragma unroll
    for (int b = 0; b < kNB; ++b) sum[b] = 0.f;
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
        const int step = g * GS + j, a = step / G::KCH, kk = step % G::KCH;
#pragma unroll
        for (int b = 0; b < kNB; ++b) {
          if (kk == 0) {
            f32x16_t z;
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = 0.f;
            sacc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][j], qf[b][kk], z, 0, 0, 0);
          } else {
            sacc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][j], qf[b][kk], sacc[a][b], 0, 0, 0);
          }
        }
      }
      if (g & 1) {
        // exponentials of quarter q of the current tile: exactly the keys of P^T fragment q
        const int q = g >> 1, ea = q >> 1, ee = q & 1;
#pragma unroll
        for (int b = 0; b < kNB; ++b) {
          float pv[8];
#pragma unroll
          for (int v = 0; v < 8; ++v) {
            pv[v] = __builtin_amdgcn_exp2f(scur[ea][b][ee * 8 + v] * c2 - mb[b]);
            sum[b] += pv[v];
          }
          u32x4_t w;
#pragma unroll
          for (int i = 0; i < 4; ++i) w[i] = pack_bf16(pv[2 * i], pv[2 * i + 1]);
          pf[b][q] = __builtin_bit_cast(bf16x8_t, w);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int b = 0; b < kNB; ++b) l_run[b] += sum[b];
  };
  // O^T += V^T P^T from V buffer BUF
  auto pv_mma = [&](auto buf_c, const bf16x8_t (&pf)[kNB][4]) {
    constexpr int BUF = decltype(buf_c)::value;
    typedef __attribute__((address_space(3))) s16x4_t lds_s16x4;
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    auto read_v = [&](int kc, int dt) {
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4 *)(smem + v_rd[dt] + (BUF * G::TILEB + kc * 16 * G::ROWB)));
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4 *)(smem + v_rd[dt] + (BUF * G::TILEB + (kc * 16 + 8) * G::ROWB)));
      const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8_t, both);
    };
    bf16x8_t fr[2][G::DT];  // V^T fragments of one 16-key step, read one step ahead
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
#pragma unroll
        for (int b = 0; b < kNB; ++b)
          oacc[dt][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[kc & 1][dt], pf[b][kc], oacc[dt][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- software-pipelined walk over the key tiles ------------------------------------------------
  // In the iteration of tile t a wave issues QK for tile t+1 together with the exponentials of
  // tile t (independent MFMA and VALU streams), then PV for tile t together with the row maxima
  // of tile t+1.  Tile t's K sits in K buffer (t - t_begin) & 1, its V in the V buffer of the
  // same parity; K for t+2 and V for t+1 are in flight meanwhile and land by the barrier.
  const int n_t = t_end - t_begin;
  if (kPipelined) {
  f32x16_t s_cur[2][kNB];
  Tile tn1;  // tile t+1 of the running iteration
  if (n_t > 0) {
    const Tile t0 = tile_of(t_begin);
    issue_k(t0, 0);
    issue_v(t0, 0);
    tn1 = t0;
    if (n_t > 1) {
      tn1 = tile_of(t_begin + 1);
      issue_k(tn1, 1);
    }
    dma_wait();
    __syncthreads();
    qk(std::integral_constant<int, 0>{}, s_cur);
    mask_and_reference(t0, s_cur);
    __syncthreads();  // every wave has read K buffer 0 before the first iteration refills it
  }
  auto body = [&](auto par_c, int t) {  // tile t, with t + 1 < t_end
    constexpr int PAR = decltype(par_c)::value;
    Tile tn2 = tn1;
    if (t + 2 < t_end) {
      tn2 = tile_of(t + 2);
      issue_k(tn2, PAR);
    }
    issue_v(tn1, PAR ^ 1);
    f32x16_t s_next[2][kNB];
    bf16x8_t pf[kNB][4];
    qk_with_exponentials(std::integral_constant<int, PAR ^ 1>{}, s_next, s_cur, pf);
    pv_mma(std::integral_constant<int, PAR>{}, pf);
    mask_and_reference(tn1, s_next);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < kNB; ++b) s_cur[a][b] = s_next[a][b];
    tn1 = tn2;
    dma_wait();
    __syncthreads();  // tiles t+2 (K) and t+1 (V) have landed; the buffers of tile t are free
  };
  auto last = [&](auto par_c) {
    constexpr int PAR = decltype(par_c)::value;
    bf16x8_t pf[kNB][4];
    exponentials(s_cur, pf);
    pv_mma(std::integral_constant<int, PAR>{}, pf);
  };
  if (n_t > 0) {
    int i = 0;
#pragma unroll 1
    for (; i + 2 < n_t; i += 2) {
      body(std::integral_constant<int, 0>{}, t_begin + i);
      body(std::integral_constant<int, 1>{}, t_begin + i + 1);
    }
    if (i + 1 < n_t) {
      body(std::integral_constant<int, 0>{}, t_begin + i);
      ++i;
    }
    if (i & 1) last(std::integral_constant<int, 1>{}); else last(std::integral_constant<int, 0>{});
  }
  } else {
    // Plain order: fill the next tile, then QK, softmax, PV of this one.  With two waves per
    // SIMD the hardware overlaps one wave's VALU phase with the other's MFMA phase.
    auto simple = [&](auto par_c, int t) {
      constexpr int PAR = decltype(par_c)::value;
      const Tile tl = tile_of(t);
      if (t + 1 < t_end) {
        const Tile tn = tile_of(t + 1);
        issue_k(tn, PAR ^ 1);
        issue_v(tn, PAR ^ 1);
      }
      f32x16_t sacc[2][kNB];
      bf16x8_t pf[kNB][4];
      qk(std::integral_constant<int, PAR>{}, sacc);
      mask_and_reference(tl, sacc);
      exponentials(sacc, pf);
      pv_mma(std::integral_constant<int, PAR>{}, pf);
      dma_wait();
      __syncthreads();
    };
    if (n_t > 0) {
      const Tile t0 = tile_of(t_begin);
      issue_k(t0, 0);
      issue_v(t0, 0);
    }
    dma_wait();  // unconditional: the Q fragment loads are then known to be complete inside the loop
    __syncthreads();
    int t = t_begin;
#pragma unroll 1
    for (; t + 1 < t_end; t += 2) {
      simple(std::integral_constant<int, 0>{}, t);
      simple(std::integral_constant<int, 1>{}, t + 1);
    }
    if (t < t_end) simple(std::integral_constant<int, 0>{}, t);
  }
  __syncthreads();  // every wave is done with the tiles before LDS is reused for staging

  // ---- epilogue: each wave transposes its O^T through its own slice of LDS, half of the head
  //      dimension at a time, so that rows leave as contiguous lines (all waves are past the
  //      loop's last barrier, and nothing else touches LDS any more) ---------------------------------
  constexpr int HD = D / 2;               // floats per staged row piece
  constexpr int HCH = HD / 4;             // 16-byte chunks per piece (16 or 8)
  constexpr int PITCH = HD * 4;           // bytes per staged row piece (256 or 128)
  constexpr int HLPR = 256 / PITCH;       // pieces per 256-byte LDS line
  lds_char *stage = smem + wave * (32 * PITCH);
  float inv[kNB], l_tot[kNB];
#pragma unroll
  for (int b = 0; b < kNB; ++b) {
    l_tot[b] = l_run[b] + other_half(l_run[b]);
    inv[b] = (p.n_splits == 1) ? 1.0f / l_tot[b] : 1.0f;
  }
#pragma unroll
  for (int b = 0; b < kNB; ++b) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      // write: lane (col, hf) owns query row `col`; chunk index XOR row keeps banks apart
#pragma unroll
      for (int dh = 0; dh < G::DT / 2; ++dh) {
        const int dt = half * (G::DT / 2) + dh;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int chunk = dh * 8 + q4 * 2 + hf;  // 16-byte chunk inside the piece
          f32x4_t w = {oacc[dt][b][q4 * 4 + 0] * inv[b], oacc[dt][b][q4 * 4 + 1] * inv[b],
                       oacc[dt][b][q4 * 4 + 2] * inv[b], oacc[dt][b][q4 * 4 + 3] * inv[b]};
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
        const int rr = pass * ROWS_PP + lane / HCH;  // row inside this 32-row group
        const int ch = lane % HCH;
        const f32x4_t w = *reinterpret_cast<const __attribute__((address_space(3))) f32x4_t *>(
            stage + rr * PITCH + ((ch ^ ((rr / HLPR) & (HCH - 1))) << 4));
        const int r = row0 + wave * kRowsPerWave + b * 32 + rr;
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
    if (p.n_splits > 1 && hf == 0 && row_ok[b]) {
      const int r = row0 + wave * kRowsPerWave + b * 32 + col;
      const int i = r / Gq;
      const int g = r - i * Gq;
      const int64_t prow = (int64_t)(pr.q_tok0 + i) * p.n_q_heads + kvh * Gq + g;
      float2 ml = {m_ref[b] == -INFINITY ? -INFINITY : mb[b], l_tot[b]};  // reference in log2 units
      *reinterpret_cast<float2 *>(p.part_ml + ((int64_t)split * p.part_rows + prow) * 2) = ml;
    }
  }
}

// Merge split partials in split order: m = max m_i, w_i = 2^(m_i - m),
// o = sum_i w_i O_i / sum_i w_i l_i.
template <int D>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(AttnParams p, int64_t n_rows) {
  constexpr int TPR = D / 4;              // threads per row
  constexpr int RPB = kCombineThreads / TPR;     // rows per workgroup
  const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / TPR;
  if (row >= n_rows) return;
  const int d = (threadIdx.x % TPR) * 4;
  float m = -INFINITY;
  for (int s = 0; s < p.n_splits; ++s) m = fmaxf(m, p.part_ml[((int64_t)s * p.part_rows + row) * 2]);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int s = 0; s < p.n_splits; ++s) {
    const float2 ml = *reinterpret_cast<const float2 *>(p.part_ml + ((int64_t)s * p.part_rows + row) * 2);
    if (ml.x == -INFINITY) continue;  // this split saw no visible key for the row
    const float w = __builtin_amdgcn_exp2f(ml.x - m);
    const f32x4_t o = *reinterpret_cast<const f32x4_t *>(p.part_o + ((int64_t)s * p.part_rows + row) * D + d);
    l += w * ml.y;
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
  const size_t lds = 4 * Geo<D>::TILEB;  // two K and two V buffers; the epilogue staging (kWaves * 32 * D * 2 bytes) fits inside
  static_assert((size_t)kWaves * 32 * D * 2 <= 4 * (size_t)Geo<D>::TILEB, "epilogue staging must fit the tile buffers");
  hipLaunchKernelGGL((attn_kernel<D, Meta>), dim3((unsigned)n_wg), dim3(kThreads), lds, stream, p, meta, rt);
  return hipGetLastError();
}

}  // namespace

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
