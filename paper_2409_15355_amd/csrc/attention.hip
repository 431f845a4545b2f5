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
//   - A workgroup (4 wavefronts) owns 256 packed query rows of one KV head.  Row
//     r = token * G + head_in_group packs the G query heads of a GQA group next to each
//     other, so one K/V tile streamed through LDS serves all of them.
//   - Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: keys
//     run along accumulator registers and queries along lanes, so the softmax max/sum
//     reduce in registers plus a single half-wave exchange, and the exponentials are
//     already in the B-operand layout of the second contraction O^T = V^T P^T.
//   - V^T fragments come straight out of the row-major V tile with the LDS transpose
//     read (ds_read_b64_tr_b16); K fragments with 16-byte reads.  Both tiles use an XOR
//     swizzle so that neither the 16-byte writes nor the fragment reads conflict.
//   - Softmax runs in fp32 in the log2 domain; P is rounded to bf16 for the second
//     MFMA; the output is rounded once.
//   - The KV range can be cut into n_splits pieces; each piece writes un-normalised
//     fp32 partials (max, sum, O) that combine_kernel merges in a fixed order.
#include "ba_device.h"

namespace ba {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kRowsPerWave = kTileRows / kWaves;  // 64 = two 32-query MFMA column groups

template <int D>
struct Geo {
  static constexpr int KCH = D / 16;          // k-steps of the QK contraction
  static constexpr int DT = D / 32;           // 32-row slabs of O^T
  static constexpr int CPR = D / 8;           // 16-byte chunks per K/V row
  static constexpr int ROWB = D * 2;          // bytes per K/V row in LDS
  static constexpr int LPR = 256 / ROWB;      // rows per 256-byte LDS line (1 or 2)
  static constexpr int GPR = ROWB / 64;       // 64-byte granules per row
  static constexpr int RPP = kThreads / CPR;  // rows loaded per pass
  static constexpr int NP = kTileKeys / RPP;  // passes per tile
  static constexpr int TILEB = kTileKeys * ROWB;
};

template <int D>
__device__ __forceinline__ int k_lds_off(int row, int chunk) {
  using G = Geo<D>;
  return row * G::ROWB + ((chunk ^ ((row / G::LPR) & (G::CPR - 1))) << 4);
}
template <int D>
__device__ __forceinline__ int v_lds_off(int row, int granule, int within) {
  using G = Geo<D>;
  return row * G::ROWB + ((granule ^ ((row / G::LPR) & (G::GPR - 1))) << 6) + within;
}

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

// Stage one K/V tile (64 rows) from global memory into registers.  Rows at or beyond
// `valid` read as zero so that masked keys give finite scores and 0 * v stays 0.
template <int D>
__device__ __forceinline__ void load_tile(u32x4_t (&reg)[Geo<D>::NP], const uint16_t *base,
                                          int64_t stride_tok, int valid) {
  using G = Geo<D>;
  const int chunk = threadIdx.x % G::CPR;
  const int row0 = threadIdx.x / G::CPR;
#pragma unroll
  for (int i = 0; i < G::NP; ++i) {
    int row = row0 + i * G::RPP;
    u32x4_t z = {0u, 0u, 0u, 0u};
    reg[i] = (row < valid)
                 ? *reinterpret_cast<const u32x4_t *>(base + (int64_t)row * stride_tok + chunk * 8)
                 : z;
  }
}
template <int D, bool IS_V>
__device__ __forceinline__ void store_tile(const u32x4_t (&reg)[Geo<D>::NP], char *lds) {
  using G = Geo<D>;
  const int chunk = threadIdx.x % G::CPR;
  const int row0 = threadIdx.x / G::CPR;
#pragma unroll
  for (int i = 0; i < G::NP; ++i) {
    int row = row0 + i * G::RPP;
    int off = IS_V ? v_lds_off<D>(row, chunk >> 2, (chunk & 3) << 4) : k_lds_off<D>(row, chunk);
    *reinterpret_cast<u32x4_t *>(lds + off) = reg[i];
  }
}

template <int D, typename Meta>
__global__ __launch_bounds__(kThreads) void attn_kernel(AttnParams p, Meta meta, RopeTable rt) {
  using G = Geo<D>;
  extern __shared__ __attribute__((aligned(256))) char smem[];
  auto ks = [&](int buf) -> char * { return smem + buf * G::TILEB; };
  auto vs = [&](int buf) -> char * { return smem + (2 + buf) * G::TILEB; };

  // ---- which work item -------------------------------------------------------------
  int id = blockIdx.x;
  const int rowtile = id % p.total_tiles;
  id /= p.total_tiles;
  const int kvh = id % p.n_kv_heads;
  const int split = id / p.n_kv_heads;
  const Problem pr = locate(meta, rowtile);

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
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
  bf16x8_t qf[2][G::KCH];
  int tok[2];       // query token (inside the problem) of this lane's two columns
  bool row_ok[2];
  int64_t o_off[2];  // element offset of the output row
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int r = row0 + wave * kRowsPerWave + b * 32 + col;
    row_ok[b] = r < n_rows;
    const int i = r / Gq;
    const int g = r - i * Gq;
    tok[b] = i;
    const int head = kvh * Gq + g;
    o_off[b] = (int64_t)(pr.q_tok0 + i) * p.o_st + (int64_t)head * p.o_sh;
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

  // ---- running softmax state and O^T accumulators ------------------------------------------
  f32x16_t oacc[G::DT][2];
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[dt][b][v] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};  // running max, raw score units
  float l_run[2] = {0.f, 0.f};              // this lane's share of the running sum
  const float c2 = p.scale_log2e;

  // tile geometry helper
  auto tile_ptrs = [&](int t, const uint16_t *&kp, const uint16_t *&vp, int64_t &kst, int64_t &vst,
                       int &valid, int &key0, bool &causal) {
    if (t < n_ctx_tiles) {
      const int64_t r0 = (int64_t)pr.ctx0 + (int64_t)t * kTileKeys;
      kp = p.kc + r0 * p.kc_st + (int64_t)kvh * p.kc_sh;
      vp = p.vc + r0 * p.vc_st + (int64_t)kvh * p.vc_sh;
      kst = p.kc_st;
      vst = p.vc_st;
      valid = min(kTileKeys, pr.tctx - t * kTileKeys);
      key0 = 0;
      causal = false;
    } else {
      const int tc = t - n_ctx_tiles;
      const int64_t r0 = (int64_t)pr.q_tok0 + (int64_t)tc * kTileKeys;
      kp = p.kf + r0 * p.kf_st + (int64_t)kvh * p.kf_sh;
      vp = p.vf + r0 * p.vf_st + (int64_t)kvh * p.vf_sh;
      kst = p.kf_st;
      vst = p.vf_st;
      valid = min(kTileKeys, pr.lq - tc * kTileKeys);
      key0 = tc * kTileKeys;
      causal = true;
    }
  };

  u32x4_t kreg[G::NP], vreg[G::NP];
  if (t_begin < t_end) {
    const uint16_t *kp, *vp;
    int64_t kst, vst;
    int valid, key0;
    bool causal;
    tile_ptrs(t_begin, kp, vp, kst, vst, valid, key0, causal);
    load_tile<D>(kreg, kp, kst, valid);
    load_tile<D>(vreg, vp, vst, valid);
    store_tile<D, false>(kreg, ks(0));
    store_tile<D, true>(vreg, vs(0));
  }
  __syncthreads();

  const int first_tok_wave = (row0 + wave * kRowsPerWave) / Gq;

#pragma unroll 1
  for (int t = t_begin; t < t_end; ++t) {
    const int cur = (t - t_begin) & 1;
    const uint16_t *kp, *vp;
    int64_t kst, vst;
    int valid, key0;
    bool causal;
    tile_ptrs(t, kp, vp, kst, vst, valid, key0, causal);

    // prefetch the next tile into registers while this one is consumed from LDS
    const bool have_next = t + 1 < t_end;
    if (have_next) {
      const uint16_t *nkp, *nvp;
      int64_t nkst, nvst;
      int nvalid, nkey0;
      bool ncausal;
      tile_ptrs(t + 1, nkp, nvp, nkst, nvst, nvalid, nkey0, ncausal);
      load_tile<D>(kreg, nkp, nkst, nvalid);
      load_tile<D>(vreg, nvp, nvst, nvalid);
    }

    // ---- S^T = K Q^T : sacc[a][b] is keys 32a..32a+31 x queries 32b..32b+31 --------------
    f32x16_t sacc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[a][b][v] = 0.f;
    const char *kl = ks(cur);
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk) {
        const int key = a * 32 + col;
        bf16x8_t kfrag = *reinterpret_cast<const bf16x8_t *>(kl + k_lds_off<D>(key, kk * 2 + hf));
        sacc[a][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag, qf[0][kk], sacc[a][0], 0, 0, 0);
        sacc[a][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag, qf[1][kk], sacc[a][1], 0, 0, 0);
      }
    }

    // ---- mask (only tiles that need it), online softmax --------------------------------------
    const bool need_mask = causal ? (key0 + kTileKeys - 1 > first_tok_wave) || (valid < kTileKeys)
                                  : (valid < kTileKeys);
    bf16x8_t pf[2][4];  // P^T fragments: [query group][16-key step]
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if (need_mask) {
        int lim = causal ? min(tok[b] - key0 + 1, valid) : valid;  // visible keys in this tile
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = a * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
            if (key >= lim) sacc[a][b][v] = -INFINITY;
          }
      }
      float mx = sacc[0][b][0];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[a][b][v]);
      mx = fmaxf(mx, other_half(mx));
      const float m_new = fmaxf(m_run[b], mx);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f((m_run[b] - m_safe) * c2);
      const float mb = m_safe * c2;
      m_run[b] = m_new;
      float sum = 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        float pv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          pv[v] = __builtin_amdgcn_exp2f(sacc[a][b][v] * c2 - mb);
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
      l_run[b] = l_run[b] * alpha + sum;
#pragma unroll
      for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][b][v] *= alpha;
    }

    // ---- O^T += V^T P^T ---------------------------------------------------------------------------
    const char *vl = vs(cur);
    const int vrow = hf * 4 + ((lane & 15) >> 2);
    const int vwithin = ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) {
#pragma unroll
      for (int dt = 0; dt < G::DT; ++dt) {
        const int r_lo = kc * 16 + vrow;
        const int r_hi = r_lo + 8;
        s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4_t __attribute__((address_space(3))) *)(vl + v_lds_off<D>(r_lo, dt, vwithin)));
        s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4_t __attribute__((address_space(3))) *)(vl + v_lds_off<D>(r_hi, dt, vwithin)));
        typedef short s16x8_t __attribute__((ext_vector_type(8)));
        s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8_t vfrag = __builtin_bit_cast(bf16x8_t, both);
        oacc[dt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfrag, pf[0][kc], oacc[dt][0], 0, 0, 0);
        oacc[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfrag, pf[1][kc], oacc[dt][1], 0, 0, 0);
      }
    }

    // ---- hand the prefetched tile to the other LDS buffer ------------------------------------------
    if (have_next) {
      store_tile<D, false>(kreg, ks(cur ^ 1));
      store_tile<D, true>(vreg, vs(cur ^ 1));
    }
    __syncthreads();
  }

  // ---- epilogue ------------------------------------------------------------------------------------
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const float l_tot = l_run[b] + other_half(l_run[b]);
    if (!row_ok[b]) continue;
    if (p.n_splits == 1) {
      const float inv = 1.0f / l_tot;
      uint16_t *op = p.o + o_off[b];
#pragma unroll
      for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d = dt * 32 + q4 * 8 + hf * 4;
          uint2 w;
          w.x = pack_bf16(oacc[dt][b][q4 * 4 + 0] * inv, oacc[dt][b][q4 * 4 + 1] * inv);
          w.y = pack_bf16(oacc[dt][b][q4 * 4 + 2] * inv, oacc[dt][b][q4 * 4 + 3] * inv);
          *reinterpret_cast<uint2 *>(op + d) = w;
        }
    } else {
      const int r = row0 + wave * kRowsPerWave + b * 32 + col;
      const int i = r / Gq;
      const int g = r - i * Gq;
      const int64_t prow = (int64_t)(pr.q_tok0 + i) * p.n_q_heads + kvh * Gq + g;
      float *po = p.part_o + ((int64_t)split * p.part_rows + prow) * D;
#pragma unroll
      for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d = dt * 32 + q4 * 8 + hf * 4;
          f32x4_t w = {oacc[dt][b][q4 * 4 + 0], oacc[dt][b][q4 * 4 + 1], oacc[dt][b][q4 * 4 + 2],
                       oacc[dt][b][q4 * 4 + 3]};
          *reinterpret_cast<f32x4_t *>(po + d) = w;
        }
      if (hf == 0) {
        float2 ml = {m_run[b] * c2, l_tot};  // max in log2 units (-inf if nothing was visible)
        *reinterpret_cast<float2 *>(p.part_ml + ((int64_t)split * p.part_rows + prow) * 2) = ml;
      }
    }
  }
}

// Merge split partials in split order: m = max m_i, w_i = 2^(m_i - m),
// o = sum_i w_i O_i / sum_i w_i l_i.
template <int D>
__global__ __launch_bounds__(kThreads) void combine_kernel(AttnParams p, int64_t n_rows) {
  constexpr int TPR = D / 4;              // threads per row
  constexpr int RPB = kThreads / TPR;     // rows per workgroup
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
  const size_t lds = 4 * Geo<D>::TILEB;
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
    constexpr int RPB = kThreads / (128 / 4);
    hipLaunchKernelGGL((combine_kernel<128>), dim3((unsigned)((n_rows + RPB - 1) / RPB)), dim3(kThreads), 0,
                       stream, p, n_rows);
  } else if (p.head_dim == 64) {
    constexpr int RPB = kThreads / (64 / 4);
    hipLaunchKernelGGL((combine_kernel<64>), dim3((unsigned)((n_rows + RPB - 1) / RPB)), dim3(kThreads), 0,
                       stream, p, n_rows);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ba
