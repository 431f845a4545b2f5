// Per-block encoding of SHORT blocks (arXiv 2409.15355, Section 2.1): the same causal attention
// inside every passage block as the main attention core computes, scheduled for key ranges of a
// few hundred tokens, where a work item is over before a deep software pipeline has filled.
//
// Mapping onto the hardware
//   - A workgroup of 4 wavefronts owns 128 packed query rows (row = token * G + head in group) of
//     one KV head of one block; a wave owns 32 of them.  Workgroups are small (48 KB of LDS at
//     head_dim 128) so that three of them share a compute unit: the latencies of one (its query
//     load, its first tiles, its output) are covered by the arithmetic of the others, not by a
//     pipeline inside the workgroup.
//   - K/V tiles of 32 keys go from memory straight into LDS (LDS-direct loads), two tiles ahead.
//     Per tile a wave computes S^T = K Q^T, the exponentials, and O^T += V^T P^T, in that order,
//     with one workgroup barrier per tile.  A wave whose rows all lie before a tile's first key
//     skips that tile's arithmetic.
//   - Arithmetic, operand layouts, softmax (reference set by the first tile, moved only to avoid
//     overflow) and rounding are those of the main core, so both give the same numbers for the
//     same rows.
#include <type_traits>

#include "ba_device.h"
#include "ba_lds.h"

namespace ba {
namespace {

constexpr int kSWaves = kShortTileRows / 32;  // 4
constexpr int kSThreads = kSWaves * 64;
constexpr int kSKeys = 32;   // keys per tile
constexpr int kSBuf = 3;     // tile buffers of each kind
constexpr float kRebaseAbove = 1099511627776.0f;  // 2^40: a tile sum beyond this moves the reference

template <int D>
struct SGeo {
  static constexpr int KCH = D / 16;          // k-steps of the QK contraction
  static constexpr int DT = D / 32;           // 32-row slabs of O^T
  static constexpr int CPR = D / 8;           // 16-byte chunks per row
  static constexpr int ROWB = D * 2;          // bytes per K/V row in LDS
  static constexpr int LPR = 256 / ROWB;      // rows per 256-byte LDS line (1 or 2)
  static constexpr int GPR = ROWB / 64;       // 64-byte granules per row
  static constexpr int TILEB = kSKeys * ROWB;
  static constexpr int RPI = 1024 / ROWB;     // rows filled by one LDS-direct wave instruction
  static constexpr int IPW = kSKeys / RPI / kSWaves;  // such instructions per wave, tile and kind
  static constexpr size_t LDS = (size_t)2 * kSBuf * TILEB;
  static_assert(IPW >= 1, "every wave takes part in a tile copy");
  static_assert((size_t)kSWaves * 32 * ROWB <= LDS, "the output staging must fit the tile buffers");
};


// Meta = EncodeMeta: a block sees its own tokens only (Section 2.1).  Meta = PromptMeta: a block's keys
// start wherever the table says -- at the block itself for a passage, at the first token of the
// prompt for its last block (Section 2.4: the lower-triangular mask with only the last block seeing
// the others); keys and queries then carry positions inside the prompt.
template <int D, typename Meta>
__global__ __launch_bounds__(kSThreads, 3) void encode_short_kernel(AttnParams p, Meta meta) {
  using G = SGeo<D>;
  constexpr bool kPrompt = std::is_same<Meta, PromptMeta>::value;
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char *smem = (lds_char *)smem_generic;
  // LDS map: buffer b = bytes [2 b TB, 2 (b + 1) TB): its K tile, then its V tile
  constexpr uint32_t TB = G::TILEB;

  // ---- which work item: consecutive items are the row tiles of one block at one KV head, and
  //      they share its K/V rows.  Workgroup ids are dealt round-robin to the 8 XCDs, so regroup
  //      them such that each XCD (and its L2) gets a contiguous run of items ---------------------
  uint32_t id = blockIdx.x;
  {
    constexpr uint32_t kXcds = 8;
    const uint32_t n_wg = gridDim.x, q = n_wg / kXcds, r = n_wg % kXcds, x = id % kXcds;
    id = x * q + min(x, r) + id / kXcds;
  }
  const uint32_t n_rowtiles = (uint32_t)p.total_tiles;
  const int kvh = (int)fast_div(id, p.tiles_div);
  // (per-block encoding: a block's long row tiles first; whole prompts: the host's order)
  const uint32_t id_lo = id - (uint32_t)kvh * n_rowtiles;
  const int rowtile = kPrompt ? (int)id_lo : (int)(n_rowtiles - 1 - id_lo);
  // block of this row tile: the largest b with tile_start[b] <= rowtile, found in three rounds of
  // independent table reads (every 32nd entry, every 4th, every one) instead of a bisection's nine
  // dependent ones: the reads are scalar loads, and a work item this short feels each round trip
  int b = 0;
  static_assert(kEncMaxBlocks <= 320, "ten coarse samples cover the table");
  {
    // (entries past the last block hold INT_MAX, so no candidate needs a bounds check)
    int hit[10];
#pragma unroll
    for (int k = 1; k < 10; ++k) hit[k] = meta.tile_start[k * 32];
#pragma unroll
    for (int k = 1; k < 10; ++k) b += hit[k] <= rowtile ? 32 : 0;
    int fine = 0;
#pragma unroll
    for (int k = 1; k < 8; ++k) hit[k] = meta.tile_start[min(b + 4 * k, kEncMaxBlocks)];
#pragma unroll
    for (int k = 1; k < 8; ++k) fine += hit[k] <= rowtile ? 4 : 0;
    b += fine;
    fine = 0;
#pragma unroll
    for (int k = 1; k < 4; ++k) hit[k] = meta.tile_start[min(b + k, kEncMaxBlocks)];
#pragma unroll
    for (int k = 1; k < 4; ++k) fine += hit[k] <= rowtile ? 1 : 0;
    b += fine;
  }
  int q_tok0, lq, k_tok0;  // the block's first token, its length, the first key it sees
  if constexpr (kPrompt) {
    q_tok0 = meta.start[b];
    lq = meta.len[b];
    k_tok0 = meta.kstart[b];
  } else {
    q_tok0 = meta.offs[b];
    lq = meta.offs[b + 1] - q_tok0;
    k_tok0 = q_tok0;
  }
  const int dq = q_tok0 - k_tok0;  // the block's first token, counted in keys
  const int lk = dq + lq;          // keys up to the block's end
  const int jt = rowtile - meta.tile_start[b];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 31;  // query column inside the 32-wide MFMA group
  const int hf = lane >> 5;   // which half of the wave
  const int Gq = p.group;
  const int n_rows = lq * Gq;
  const int row0 = jt * kShortTileRows;

  // key tiles of the workgroup (up to its last row's token) and of this wave
  const int last_row = min(n_rows, row0 + kShortTileRows) - 1;
  const int n_t = (dq + (int)fast_div((uint32_t)last_row, p.group_div)) / kSKeys + 1;
  const int wave_row0 = row0 + wave * 32;
  const int wave_last_row = min(n_rows, wave_row0 + 32) - 1;
  const int wave_n_t =
      wave_last_row >= wave_row0 ? (dq + (int)fast_div((uint32_t)wave_last_row, p.group_div)) / kSKeys + 1 : 0;
  const int first_tok_wave = (int)fast_div((uint32_t)wave_row0, p.group_div);
  const int first_key_wave = dq + first_tok_wave;  // the key that is the wave's first token

  const int my_row = wave_row0 + col;
  const int my_tok = (int)fast_div((uint32_t)my_row, p.group_div);
  const int my_key = dq + my_tok;  // the key that is this lane's token: the last one it sees

  // ---- Q rows (B operand of S^T = K Q^T) and, if they are to be rotated, the rows of the pre-pass's
  //      table of scale * log2(e) * (cos, sin) for this wave's tokens: requested first and all at
  //      once, so that the set-up below runs under their latency.  Both arrive as whole rows (a
  //      lane fetching only its own 16 bytes of a row would cost a cache line each); the Q rows are
  //      then turned into the fragment layout (lane = row) through this wave's slice of LDS ---------
  // (rows beyond the block's take its last row: finite numbers that are never stored)
  constexpr int QRPI = 64 / G::CPR;  // Q rows per load instruction
  static_assert(32 / QRPI == G::KCH, "as many row loads as fragments");
  u32x4_t ld[G::KCH];
  constexpr uint32_t TROW = D * 4;    // bytes of a table row
  constexpr int TCH = TROW / 16;      // its 16-byte chunks
  constexpr int kTabOps = 8 * TROW / 1024;  // LDS-direct loads per wave for 8 table rows
  static_assert(kSBuf == 3, "tile buffers 0 and 1 take the first tiles, 2 the waves' slices");
  static_assert(kSWaves * 8 * TROW <= 2 * TB, "the table slices fit one tile buffer");
  static_assert(kSWaves * 16 * G::ROWB <= 2 * TB, "the Q slices (16 rows at a time) fit one tile buffer");
  static_assert(16 * G::ROWB == 8 * TROW, "one slice serves both uses");
  const uint32_t tab_ofs = 2 * (2 * TB) + wave * (8 * TROW);  // first the table rows ...
  const uint32_t q_ofs = tab_ofs;                              // ... then, once those are in registers, Q rows
  int tab_tl = 0;  // this lane's row of the table slice
  // Whole rows move QRPI at a time: this lane's row in step u is wave_row0 + u * QRPI + lane / CPR and
  // its piece chunk lane % CPR.  Its element offset tok * st + g * sh (relative to the block's first
  // token and the group's first head; 32 bits by the host's check) is carried from step to step:
  // four rows on is either four heads on or, past the group's last head, into the next token.
  // (worked out afresh by each of the two walks, load and store: kept, the row numbers would occupy
  // registers all through the tile loop)
  auto walk_rows = [&](int ln, uint32_t st, uint32_t sh, auto &&visit) __attribute__((always_inline)) {
    const int wr_r0 = wave_row0 + ln / G::CPR;
    const int wr_tok0 = (int)fast_div((uint32_t)wr_r0, p.group_div);
    const int wr_g0 = wr_r0 - wr_tok0 * Gq;
    uint32_t off = (uint32_t)wr_tok0 * st + (uint32_t)wr_g0 * sh;
    int g = wr_g0;
    const uint32_t d_in = 4u * sh, d_wrap = st + (uint32_t)(4 - Gq) * sh;
#pragma unroll
    for (int u = 0; u < G::KCH; ++u) {
      visit(u, off, wr_r0);
#pragma unroll
      for (int s4 = 0; s4 < QRPI / 4; ++s4) {
        g += 4;
        const bool wrap = g >= Gq;
        g = wrap ? g - Gq : g;
        off += wrap ? d_wrap : d_in;
      }
    }
  };
  {
    const char *qbase = (const char *)(p.q + (int64_t)q_tok0 * p.q_st + (int64_t)(kvh * Gq) * p.q_sh);
    const uint32_t q_st = (uint32_t)p.q_st, q_sh = (uint32_t)p.q_sh;
    const uint32_t last_off = (uint32_t)(lq - 1) * q_st + (uint32_t)(Gq - 1) * q_sh;  // the block's last row
    walk_rows(lane, q_st, q_sh, [&](int u, uint32_t off, int wr_r0) __attribute__((always_inline)) {
      const uint32_t o = wr_r0 < n_rows - u * QRPI ? off : last_off;
      ld[u] = *reinterpret_cast<const u32x4_t *>(qbase + (o * 2u + (uint32_t)(lane % G::CPR) * 16u));
    });
    if (p.q_table) {
      // The rows of a wave span at most 8 tokens (the host sends only groups of 4 or more query
      // heads here).  Chunk c of token row t sits at chunk c ^ (t & 7), which keeps the reads of
      // different tokens off each other's banks.
      // (a row per token of the call, or, for per-block encoding, a row per position inside the block)
      const char *tbase = (const char *)(p.q_table + (p.q_table_by_pos ? (int64_t)0 : (int64_t)q_tok0 * D));
#pragma unroll
      for (int u = 0; u < kTabOps; ++u) {
        const int t = u * (1024 / TROW) + lane / TCH, pc = lane % TCH;
        const uint32_t tok = (uint32_t)min(first_tok_wave + t, lq - 1);
        lds_dma16(tbase, tok * TROW + (uint32_t)((pc ^ (t & 7)) << 4), (uint32_t)(uintptr_t)smem + tab_ofs + u * 1024);
      }
      const int ld_tok = (int)fast_div((uint32_t)min(my_row, n_rows - 1), p.group_div);
      tab_tl = max(ld_tok - first_tok_wave, 0);
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- per-lane LDS read offsets inside a tile buffer (same swizzles as the tile fill below) ----
  uint32_t k_rd[G::KCH];  // K fragment: row `col`, chunk 2 kk + hf
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

  // ---- tile fill: one wave instruction fills 1024 contiguous LDS bytes, lane i writing
  //      [16 i, 16 i + 16); the swizzle is applied on the global side.  Rows at or beyond a tile's
  //      valid count re-read its last valid row: their scores are masked, and a finite duplicate
  //      keeps 0 * v equal to 0 ------------------------------------------------------------------
  const char *k_base = (const char *)(p.kf + (int64_t)k_tok0 * p.kf_st + (int64_t)kvh * p.kf_sh);
  const char *v_base = (const char *)(p.vf + (int64_t)k_tok0 * p.vf_st + (int64_t)kvh * p.vf_sh);
  const uint32_t k_rb = (uint32_t)p.kf_st * 2u, v_rb = (uint32_t)p.vf_st * 2u;  // row strides, bytes
  int c_row[G::IPW];
  uint32_t c_kchunk[G::IPW], c_vchunk[G::IPW];
#pragma unroll
  for (int u = 0; u < G::IPW; ++u) {
    const int row = (wave * G::IPW + u) * G::RPI + lane / G::CPR, pos = lane % G::CPR;
    c_row[u] = row;
    c_kchunk[u] = (uint32_t)(pos ^ ((row / G::LPR) & (G::CPR - 1))) << 4;
    c_vchunk[u] = (uint32_t)((((pos >> 2) ^ ((row / G::LPR) & (G::GPR - 1))) << 2) | (pos & 3)) << 4;
  }
  const uint32_t lds_copy = (uint32_t)(uintptr_t)smem + wave * G::IPW * 1024;
  auto issue_copy = [&](int t, int buf) __attribute__((always_inline)) {
    const int valid = min(kSKeys, lk - t * kSKeys);
    const char *kp = k_base + (uint64_t)(uint32_t)(t * kSKeys) * (uint64_t)k_rb;
    const char *vp = v_base + (uint64_t)(uint32_t)(t * kSKeys) * (uint64_t)v_rb;
#pragma unroll
    for (int u = 0; u < G::IPW; ++u) {
      const uint32_t row = (uint32_t)min(c_row[u], valid - 1);
      lds_dma16(kp, row * k_rb + c_kchunk[u], lds_copy + (uint32_t)buf * (2 * TB) + u * 1024);
      lds_dma16(vp, row * v_rb + c_vchunk[u], lds_copy + (uint32_t)buf * (2 * TB) + TB + u * 1024);
    }
  };
  constexpr int kOpsPerTile = 2 * G::IPW;  // vector-memory operations of one wave per tile
  issue_copy(0, 0);  // (buffer 2 holds the waves' slices until the first barrier)
  if (1 < n_t) issue_copy(1, 1);
  __builtin_amdgcn_sched_barrier(0);  // the copies go out before anything waits for the Q rows

  // ---- rotate (or just scale) the Q rows into the fragments ---------------------------------------
  dma_wait<0>();  // the table rows and the first tile (this wave's share) have landed
  // The table first: entry j of a table row = (cos, sin) of pair j.  Interleaved pairs: fragment kk
  // holds pairs kk * 8 + hf * 4 + (0..3); half-split pairs: fragments kk and kk + KCH/2 hold dims
  // kk * 16 + hf * 8 + (0..7) and their partners, i.e. pairs of those same numbers.
  f32x4_t cs[2 * G::KCH];
  if (p.q_table) {
    const bool halves = p.rope_layout != 0;
#pragma unroll
    for (int j = 0; j < 2 * G::KCH; ++j) {
      const int c = halves ? (j / 4) * 8 + (j & 3) + hf * 4 : (j / 2) * 4 + (j & 1) + hf * 2;
      cs[j] = *reinterpret_cast<const __attribute__((address_space(3))) f32x4_t *>(
          smem + tab_ofs + (uint32_t)(tab_tl * TROW + ((c ^ (tab_tl & 7)) << 4)));
    }
  }
  // whole rows -> fragments: 16 rows at a time through the slice (LDS serves a wave's accesses in
  // order, so the slice needs no barrier); every lane reads the chunks of row `col mod 16` in both
  // passes and keeps those of the pass its row was in
  u32x4_t raw[G::KCH];
  {
    u32x4_t got[2][G::KCH];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
      for (int u = 0; u < G::KCH / 2; ++u) {
        const int rp = u * QRPI + lane / G::CPR, c = lane % G::CPR;
        *reinterpret_cast<__attribute__((address_space(3))) u32x4_t *>(
            smem + q_ofs + rp * G::ROWB + ((c ^ (rp & (G::CPR - 1))) << 4)) = ld[pass * (G::KCH / 2) + u];
      }
      const int rp = col & 15;
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk)
        got[pass][kk] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t *>(
            smem + q_ofs + rp * G::ROWB + (((kk * 2 + hf) ^ (rp & (G::CPR - 1))) << 4));
    }
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk)
#pragma unroll
      for (int e = 0; e < 4; ++e) raw[kk][e] = (col >> 4) ? got[1][kk][e] : got[0][kk][e];
  }
  bf16x8_t qf[G::KCH];
  if (p.q_table) {
    const bool halves = p.rope_layout != 0;
    if (!halves) {
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk) {
        const f32x4_t cs0 = cs[2 * kk], cs1 = cs[2 * kk + 1];
        const float c[4] = {cs0[0], cs0[2], cs1[0], cs1[2]}, sn[4] = {cs0[1], cs0[3], cs1[1], cs1[3]};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x = bf16_lo(raw[kk][e]), y = bf16_hi(raw[kk][e]);
          raw[kk][e] = pack_bf16(c[e] * x - sn[e] * y, sn[e] * x + c[e] * y);
        }
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < G::KCH / 2; ++kk) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const f32x4_t t = cs[4 * kk + e];  // pairs kk * 16 + hf * 8 + 2 e and the next
          const float c0 = t[0], s0 = t[1], c1 = t[2], s1 = t[3];
          const uint32_t wa = raw[kk][e], wb = raw[kk + G::KCH / 2][e];
          const float xa0 = bf16_lo(wa), xa1 = bf16_hi(wa), xb0 = bf16_lo(wb), xb1 = bf16_hi(wb);
          raw[kk][e] = pack_bf16(c0 * xa0 - s0 * xb0, c1 * xa1 - s1 * xb1);
          raw[kk + G::KCH / 2][e] = pack_bf16(s0 * xa0 + c0 * xb0, s1 * xa1 + c1 * xb1);
        }
      }
    }
  } else if (!p.q_ready) {
    const float c2 = p.scale_log2e;
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk)
#pragma unroll
      for (int e = 0; e < 4; ++e) raw[kk][e] = pack_bf16(bf16_lo(raw[kk][e]) * c2, bf16_hi(raw[kk][e]) * c2);
  }
#pragma unroll
  for (int kk = 0; kk < G::KCH; ++kk) {
    asm volatile("" : "+v"(raw[kk]));  // the loads are waited for here, not inside the loop
    qf[kk] = __builtin_bit_cast(bf16x8_t, raw[kk]);
  }

  // ---- running state -----------------------------------------------------------------------------
  f32x16_t oacc[G::DT];
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
  float mb = 0.f;     // the row's reference, log2 units
  float l_run = 0.f;  // this lane's share of the running sum of exponentials

  auto row_max = [&](const f32x16_t &s) __attribute__((always_inline)) {
    float m0 = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) m0 = fmaxf(m0, s[v]);
    return fmaxf(m0, other_half(m0));
  };
  // P = 2^S' rounded to bf16 (the B operand of PV); returns this lane's fp32 sum of the exponentials
  auto exponentials = [&](const f32x16_t &s, bf16x8_t (&pf)[2]) __attribute__((always_inline)) {
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      u32x4_t w;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p0 = __builtin_amdgcn_exp2f(s[e * 8 + 2 * i]);
        const float p1 = __builtin_amdgcn_exp2f(s[e * 8 + 2 * i + 1]);
        s0 += p0;
        s1 += p1;
        w[i] = pack_bf16(p0, p1);
      }
      pf[e] = __builtin_bit_cast(bf16x8_t, w);
    }
    return s0 + s1;
  };

  // ---- the walk over the key tiles: tile i lives in buffer i % 3.  The barrier at the head of
  //      iteration i says two things: every wave's share of tile i has landed, and every wave is
  //      done with tile i-1 (at i = 0: with its slice of buffer 2), so the copy of tile i+2 may
  //      overwrite that buffer ------------------------------------------------------------------------
  int buf = 0;
#pragma unroll 1
  for (int i = 0; i < n_t; ++i) {
    if (i + 1 < n_t) dma_wait<kOpsPerTile>(); else dma_wait<0>();  // tile i + 1 may still be on its way
    wg_barrier();
    if (i + 2 < n_t) issue_copy(i + 2, buf == 0 ? 2 : buf - 1);
    if (i < wave_n_t) {
      const uint32_t kofs = (uint32_t)buf * (2 * TB), vofs = kofs + TB;
      // S'^T = K Q'^T - reference: the accumulator starts at minus the row's reference, so the MFMA
      // result is directly the base-2 exponent
      f32x16_t sacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[v] = -mb;
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk) {
        const bf16x8_t kfrag = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(smem + (k_rd[kk] + kofs));
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag, qf[kk], sacc, 0, 0, 0);
      }
      // mask (diagonal and ragged tiles only); all branches are wave-uniform
      const int key0 = i * kSKeys;
      const int valid = min(kSKeys, lk - key0);
      if (key0 + kSKeys - 1 > first_key_wave || valid < kSKeys) {
        const int lim = min(my_key - key0 + 1, valid);  // visible keys in this tile
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = (v >> 2) * 8 + hf * 4 + (v & 3);
          if (key >= lim) sacc[v] = -INFINITY;
        }
      }
      if (i == 0) {
        // the first tile sets the reference: its row maximum whatever the sign (nothing visible:
        // stay at 0), so a row's largest exponential so far is exactly 1
        const float mx = row_max(sacc);
        const float shift = mx == -INFINITY ? 0.f : mx;
        mb = shift;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] -= shift;
      }
      bf16x8_t pf[2];
      float tsum = exponentials(sacc, pf);
      if (__builtin_amdgcn_ballot_w64(!(tsum < kRebaseAbove)) != 0) {  // overflow guard: practically never
        asm volatile("" ::: "memory");
        const float shift = fmaxf(row_max(sacc), 0.f);  // only ever raise the reference here
        const float alpha = __builtin_amdgcn_exp2f(-shift);
        mb += shift;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] -= shift;
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
        tsum = exponentials(sacc, pf);
      }
      l_run += tsum;
      // O^T += V^T P^T
#pragma unroll
      for (int kc = 0; kc < 2; ++kc)
#pragma unroll
        for (int dt = 0; dt < G::DT; ++dt) {
          typedef __attribute__((address_space(3))) s16x4_t lds_s16x4;
          typedef short s16x8_t __attribute__((ext_vector_type(8)));
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + (v_rd[dt] + vofs) + kc * 16 * G::ROWB));
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + (v_rd[dt] + vofs) + (kc * 16 + 8) * G::ROWB));
          const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, both), pf[kc], oacc[dt], 0, 0, 0);
        }
    }
    buf = buf == kSBuf - 1 ? 0 : buf + 1;
  }

  // ---- epilogue: normalise, round once to bf16, and transpose each wave's O^T through its own
  //      slice of LDS so that rows leave as contiguous lines.  The slices lie in the tile buffers:
  //      every wave must be done with the last tile first -----------------------------------------
  // (all of this wave's LDS reads were consumed by its MFMAs, so only the barrier is needed)
  wg_barrier();
  // (lane-dependent addresses are worked out from here on, not carried through the loop in registers)
  int ln = lane;
  asm volatile("" : "+v"(ln));
  const int ecol = ln & 31, ehf = ln >> 5;
  lds_char *stage = smem + wave * (32 * G::ROWB);
  const float l_tot = l_run + other_half(l_run);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      // dims dt * 32 + q4 * 8 + hf * 4 + (0..3) of query row `col`
      const int col = ecol, hf = ehf;
      const int chunk = dt * 4 + q4;
      typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
      u32x2_t w;
      w[0] = pack_bf16(oacc[dt][q4 * 4 + 0] * inv, oacc[dt][q4 * 4 + 1] * inv);
      w[1] = pack_bf16(oacc[dt][q4 * 4 + 2] * inv, oacc[dt][q4 * 4 + 3] * inv);
      *reinterpret_cast<__attribute__((address_space(3))) u32x2_t *>(
          stage + col * G::ROWB + ((chunk ^ (col & (G::CPR - 1))) << 4) + hf * 8) = w;
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  {
    // (all the pieces are read back before the first store, so that the stores do not each wait
    // for their own read)
    u32x4_t w[G::KCH];
#pragma unroll
    for (int u = 0; u < G::KCH; ++u) {
      const int rr = u * QRPI + ln / G::CPR;  // row inside this wave's 32
      const int ch = ln % G::CPR;
      w[u] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t *>(
          stage + rr * G::ROWB + ((ch ^ (rr & (G::CPR - 1))) << 4));
    }
    char *obase = (char *)(p.o + (int64_t)q_tok0 * p.o_st + (int64_t)(kvh * Gq) * p.o_sh);
    walk_rows(ln, (uint32_t)p.o_st, (uint32_t)p.o_sh, [&](int u, uint32_t off, int wr_r0) __attribute__((always_inline)) {
      if (wr_r0 < n_rows - u * QRPI)
        *reinterpret_cast<u32x4_t *>(obase + (off * 2u + (uint32_t)(ln % G::CPR) * 16u)) = w[u];
    });
  }
  // the row's log-sum-exp of its scaled scores (natural logarithm), for a backward pass
  if (p.lse != nullptr && ehf == 0 && wave_row0 + ecol < n_rows) {
    const int r = wave_row0 + ecol;
    const int tok = (int)fast_div((uint32_t)r, p.group_div);
    p.lse[(int64_t)(q_tok0 + tok) * p.n_q_heads + kvh * Gq + (r - tok * Gq)] =
        (mb + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;  // (v_log_f32 is the base-2 logarithm)
  }
}

template <int D, typename Meta>
hipError_t launch_short_t(const AttnParams &p, const Meta &meta, hipStream_t stream) {
  const int64_t n_wg = (int64_t)p.total_tiles * p.n_kv_heads;
  if (n_wg == 0) return hipSuccess;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  static_assert(SGeo<D>::LDS <= 64 * 1024, "fits the default dynamic LDS limit");
  hipLaunchKernelGGL((encode_short_kernel<D, Meta>), dim3((unsigned)n_wg), dim3(kSThreads), SGeo<D>::LDS, stream, p,
                     meta);
  return hipGetLastError();
}

}  // namespace


hipError_t launch_attn_encode_short(const AttnParams &p, const EncodeMeta &meta, hipStream_t stream) {
  if (p.n_splits != 1) return hipErrorInvalidValue;
  if (p.head_dim == 128) return launch_short_t<128, EncodeMeta>(p, meta, stream);
  if (p.head_dim == 64) return launch_short_t<64, EncodeMeta>(p, meta, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_attn_prompt_short(const AttnParams &p, const PromptMeta &meta, hipStream_t stream) {
  if (p.n_splits != 1) return hipErrorInvalidValue;
  if (p.head_dim == 128) return launch_short_t<128, PromptMeta>(p, meta, stream);
  if (p.head_dim == 64) return launch_short_t<64, PromptMeta>(p, meta, stream);
  return hipErrorInvalidValue;
}

}  // namespace ba
