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
//     (global_load_lds_dwordx4), three tiles ahead of their use.
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
//   - The two waves of a SIMD run half a period apart ("ping-pong"): while one is in its
//     exponentials (VALU), the other is in its MFMA block (PV of this tile, QK of the next).
//   - The KV range can be cut into n_splits pieces; each piece writes its own normalised output
//     (fp16) with its reference and sum (fp32), and combine_kernel merges them in a fixed order.
#include <atomic>
#include <type_traits>

#include "ba_device.h"
#include "ba_lds.h"
#include "ba_schedule.h"

namespace ba {
namespace {

constexpr int kCombineThreads = 256;
constexpr int kWaves = kTileRows / 32;  // 8: each wave owns one 32-query MFMA column group
constexpr int kThreads = kWaves * 64;
constexpr int kXcds = 8;        // MI355X: workgroup ids go round-robin over 8 XCDs
constexpr int kNumKBuf = 4;     // K tiles resident in LDS
constexpr int kNumVBuf = 4;     // V tiles resident in LDS
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
  int q_tok0;     // first query token (row of q / o / kf / vf)
  int lq;         // query tokens
  int ctx0;       // first context row (contiguous context)
  int tctx;       // context rows (contiguous context)
  int blk0, blk1; // cached blocks of the context (block table)
  int ctx_tiles;  // key tiles of the context
  int jt;         // row tile inside the problem
};

__device__ __forceinline__ Problem locate(const EncodeMeta &m, int tile) {
  int b = find_segment(m.tile_start, m.n, tile);
  Problem pr;
  pr.q_tok0 = m.offs[b];
  pr.lq = m.offs[b + 1] - m.offs[b];
  pr.ctx0 = 0;
  pr.tctx = 0;
  pr.blk0 = pr.blk1 = 0;
  pr.ctx_tiles = 0;
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
  pr.blk0 = pr.blk1 = 0;
  pr.ctx_tiles = (pr.tctx + kTileKeys - 1) / kTileKeys;
  pr.jt = tile - m.tile_start[n];
  return pr;
}
template <int NP, int NB>
__device__ __forceinline__ Problem locate(const FinalBlocksMetaT<NP, NB> &m, int tile) {
  int n = find_segment(m.tile_start, m.n, tile);
  Problem pr;
  pr.q_tok0 = m.cu_q[n];
  pr.lq = m.cu_q[n + 1] - m.cu_q[n];
  pr.ctx0 = 0;
  pr.tctx = 0;
  pr.blk0 = m.cu_blk[n];
  pr.blk1 = m.cu_blk[n + 1];
  pr.ctx_tiles = m.ctx_tiles[n];
  pr.jt = tile - m.tile_start[n];
  return pr;
}


template <int D, typename Meta>
__global__ __launch_bounds__(kThreads) void attn_kernel(AttnParams p, Meta meta) {
  using G = Geo<D>;
  // context = table of cached blocks
  constexpr bool kBlocks = std::is_same<Meta, FinalBlocksMeta>::value || std::is_same<Meta, FinalBlocksMetaSmall>::value;
  constexpr bool kFinal = std::is_same<Meta, FinalMeta>::value || kBlocks;
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char *smem = (lds_char *)smem_generic;
  // LDS map: kNumKBuf K buffers from byte 0, then kNumVBuf V buffers, TILEB bytes each.
  constexpr uint32_t TB = G::TILEB;
  constexpr uint32_t VBASE = kNumKBuf * TB;

  // ---- which work item -------------------------------------------------------------------
  uint32_t id = blockIdx.x;
  if (kFinal) {
    // Consecutive work items share K/V tiles (same KV head and split, different row tile);
    // the dispatcher deals workgroup ids round-robin to the XCDs, so regroup ids such that
    // each XCD (and its L2) gets a contiguous run of work items.
    id = work_item_of_workgroup(id, gridDim.x, p.xcd_runs);
  }
  // (divisions by launch constants: multipliers from the host instead of hardware divisions, each of
  // which is some thirty instructions on the one scalar unit that the eight waves of a workgroup share)
  const ItemOrder order = {p.total_tiles, p.n_kv_heads, p.n_splits, p.kv_group};
  const ItemCoords item = item_coords(id, order, &p.item_divs);
  const int rowtile = kFinal ? item.rowtile : p.total_tiles - 1 - item.rowtile;
  const int split = item.split, kvh = item.kvh;
  const Problem pr = locate(meta, rowtile);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform, lives in an SGPR
  const int col = lane & 31;  // query column inside the 32-wide MFMA group
  const int hf = lane >> 5;   // which half of the wave
  const int Gq = p.group;
  const int n_rows = pr.lq * Gq;
  const int row0 = pr.jt * kTileRows;
  // Probe (ba_measure_xcd_speed, ba_diag_final_block_phases): which XCD this workgroup runs on, its
  // shader-clock and real-time (100 MHz) counters here and behind the walk (their ratio is the XCD's
  // clock under this load), and the real-time counter at the phase boundaries in between.
  constexpr bool kProbe = std::is_same<Meta, FinalMeta>::value;
  auto probe_mark = [&](int slot) __attribute__((always_inline)) {
    if (kProbe && p.wg_clock && threadIdx.x == 0)
      p.wg_clock[(size_t)blockIdx.x * kProbeRecord + slot] = (unsigned long long)wall_clock64();
  };
  if (kProbe && p.wg_clock && threadIdx.x == 0) {
    unsigned long long *rec = p.wg_clock + (size_t)blockIdx.x * kProbeRecord;
    rec[0] = (unsigned long long)(__builtin_amdgcn_s_getreg(6164) & 15);  // HW_REG_XCC_ID, bits 3:0
    rec[1] = (unsigned long long)clock64();
    rec[2] = (unsigned long long)wall_clock64();
  }

  // ---- key tiles this work item walks ---------------------------------------------------
  // The key range is a list of segments: fully visible context segments first (one for a
  // contiguous context, one per cached block with a block table), then the causal segment (the
  // problem's own keys).  Tiles never straddle segments.
  const int n_ctx_tiles = pr.ctx_tiles;
  const int n_ctx_segs = kBlocks ? pr.blk1 - pr.blk0 : (n_ctx_tiles > 0 ? 1 : 0);
  const int last_row = min(n_rows, row0 + kTileRows) - 1;
  const int last_tok = (int)fast_div((uint32_t)last_row, p.group_div);
  const int n_causal_tiles = causal_key_tiles(last_tok, kTileKeys);
  // this split's share of the walk (the arithmetic is the host planner's: one definition)
  const TileRange tr = split_tile_range(n_ctx_tiles, n_causal_tiles, p.n_splits, split, p.use_cuts ? p.split_cut[kvh] : nullptr,
                                        &p.split_divs);
  const int t_begin = tr.begin, t_end = tr.end;
  const int n_t = t_end - t_begin;

  const int my_row = row0 + wave * 32 + col;
  const bool row_ok = my_row < n_rows;
  // A wave none of whose 32 rows exists (the last row tile of a problem, a final block of few tokens)
  // still copies its share of the tiles and meets every barrier, but skips its exponentials and MFMAs:
  // they would run on zeros at full power, and this part's clock is set by the power it draws.
  // (not with a block table: that kernel has no scalar register left for the flag and would spill)
  const bool wave_has_rows = kBlocks || row0 + wave * 32 < n_rows;
  const int my_tok = (int)fast_div((uint32_t)my_row, p.group_div);  // query token (inside the problem) of this lane's column
  bf16x8_t qf[G::KCH];  // Q fragments, filled below once the first tile copies are on their way

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
  // Waves 0..3 fetch the K tiles and waves 4..7 the V tiles (see the walk below), so each wave
  // works out the addressing of one kind only (tensor and strides are picked first, the 64-bit
  // products come after: half as many of them).
  const bool role_b = wave >= kWaves / 2;
  const uint16_t *c_ptr = role_b ? p.vc : p.kc, *f_ptr = role_b ? p.vf : p.kf;
  const int64_t c_st = role_b ? p.vc_st : p.kc_st, c_sh = role_b ? p.vc_sh : p.kc_sh;
  const int64_t f_st = role_b ? p.vf_st : p.kf_st, f_sh = role_b ? p.vf_sh : p.kf_sh;
  const char *c_base = (const char *)(c_ptr + (int64_t)pr.ctx0 * c_st + (int64_t)kvh * c_sh);    // context segment
  const char *f_base = (const char *)(f_ptr + (int64_t)pr.q_tok0 * f_st + (int64_t)kvh * f_sh);  // causal segment
  const uint32_t c_rb = (uint32_t)c_st * 2u, f_rb = (uint32_t)f_st * 2u;  // row strides, bytes
  // Full tiles of segments with the "primary" row stride (the context's if there is one, else the
  // causal segment's) take a short path with cached lane offsets.
  const uint32_t prim_rb = n_ctx_segs > 0 ? c_rb : f_rb;
  // this lane's source row (inside the tile) and chunk offset (inside the row) for its i-th piece
  auto copy_row = [&](int i) __attribute__((always_inline)) {
    return ((wave & (kWaves / 2 - 1)) * G::IPW + i) * G::RPI + lane / G::CPR;
  };
  auto copy_chunk = [&](int i) __attribute__((always_inline)) {
    const int row = copy_row(i), pos = lane % G::CPR;
    const uint32_t kchunk = (uint32_t)(pos ^ ((row / G::LPR) & (G::CPR - 1))) << 4;
    const uint32_t vchunk = (uint32_t)((((pos >> 2) ^ ((row / G::LPR) & (G::GPR - 1))) << 2) | (pos & 3)) << 4;
    return role_b ? vchunk : kchunk;
  };
  uint32_t g_src[G::IPW];  // full per-lane byte offsets inside a full tile of primary stride
#pragma unroll
  for (int i = 0; i < G::IPW; ++i) g_src[i] = (uint32_t)copy_row(i) * prim_rb + copy_chunk(i);
  const uint32_t lds_copy =
      (uint32_t)(uintptr_t)smem + (role_b ? VBASE : 0u) + (wave & (kWaves / 2 - 1)) * G::IPW * 1024;

  // segment s of this problem: rows that exist, key tiles walked, first row (of this wave's kind)
  auto seg_len = [&](int sg) __attribute__((always_inline)) {
    if (sg >= n_ctx_segs) return pr.lq;
    if constexpr (kBlocks) return (int)meta.blk_len[pr.blk0 + sg];
    return pr.tctx;
  };
  auto seg_base = [&](int sg) __attribute__((always_inline)) {
    if (sg >= n_ctx_segs) return f_base;
    if constexpr (kBlocks) return c_base + (uint64_t)(uint32_t)meta.blk_off[pr.blk0 + sg] * (uint64_t)c_rb;
    return c_base;
  };
  // Position in the walk: segment, tile inside it, tiles left in it (this one included), plus the
  // segment's row count and first row (of this wave's kind), fetched once per segment so that the
  // loop itself never reads the tables (a scalar load would also wait for the LDS reads in flight).
  struct Cursor {
    int seg, ts, rem, len;
    const char *base;
  };
  auto enter = [&](Cursor &c, int sg, int ts) __attribute__((always_inline)) {
    c.seg = sg;
    c.ts = ts;
    c.len = seg_len(sg);
    c.base = seg_base(sg);
    c.rem = (sg >= n_ctx_segs ? n_causal_tiles : (c.len + kTileKeys - 1) / kTileKeys) - ts;
  };
  auto cursor_at = [&](int t) __attribute__((always_inline)) {
    Cursor c;
    if (t >= n_ctx_tiles) {
      enter(c, n_ctx_segs, t - n_ctx_tiles);
    } else if constexpr (kBlocks) {
      int lo = pr.blk0, hi = pr.blk1;  // largest block whose first tile is <= t
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (meta.blk_tile0[mid] <= t) lo = mid; else hi = mid;
      }
      enter(c, lo - pr.blk0, t - meta.blk_tile0[lo]);
    } else {
      enter(c, 0, t);
    }
    return c;
  };
  auto advance = [&](Cursor &c) __attribute__((always_inline)) {
    ++c.ts;
    --c.rem;
    if (c.rem == 0 && c.seg < n_ctx_segs) {  // (the host drops empty blocks: a segment has a tile)
      asm volatile("" ::: "memory");
      enter(c, c.seg + 1, 0);
    }
  };
  // Copy of the tile under a cursor into buffer `buf` of this wave's kind: a wave-uniform
  // preparation and IPW wave instructions, kept apart so that the instructions can be spread over
  // the gaps of an MFMA stream.
  struct CopyJob {
    const char *ptr;  // first row of the tile
    uint32_t dst;     // LDS byte address of this wave's first 1 KB piece
    uint32_t rb;      // row stride, bytes
    int valid;        // rows of the tile that exist
    bool full;        // all rows exist and the stride is the primary one: cached lane offsets
  };
  auto copy_prepare = [&](const Cursor &c, int buf) __attribute__((always_inline)) {
    CopyJob j;
    j.dst = lds_copy + (uint32_t)buf * TB;
    j.rb = c.seg >= n_ctx_segs ? f_rb : c_rb;
    j.ptr = c.base + (uint64_t)(uint32_t)c.ts * (uint64_t)(j.rb * (uint32_t)kTileKeys);
    j.valid = min(kTileKeys, c.len - c.ts * kTileKeys);
    j.full = j.valid == kTileKeys && j.rb == prim_rb;
    return j;
  };
  auto copy_part = [&](const CopyJob &c, int i) __attribute__((always_inline)) {
    if (c.full) {
      lds_dma16(c.ptr, g_src[i], c.dst + i * 1024);
    } else {
      asm volatile("" ::: "memory");
      lds_dma16(c.ptr, (uint32_t)min(copy_row(i), c.valid - 1) * c.rb + copy_chunk(i), c.dst + i * 1024);
    }
  };

  // ---- running state -----------------------------------------------------------------------------
  f32x16_t oacc[G::DT];
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
  float mb = 0.f;      // the row's reference, log2 units
  // minus the reference in all sixteen registers of an accumulator tuple: what the score accumulators
  // start from.  Kept (not rebuilt from mb by sixteen moves inside every MFMA block, where each vector
  // instruction of this wave delays the next MFMA) and rebuilt only when the reference moves.
  // (not with a block table: that kernel has no sixteen registers to spare and would spill them)
  constexpr bool kKeepNegmb = !kBlocks;
  f32x16_t negmb;
  auto set_negmb = [&]() __attribute__((always_inline)) {
    if constexpr (kKeepNegmb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) negmb[v] = -mb;
      asm volatile("" : "+v"(negmb));  // (opaque: or the compiler re-derives the tuple from mb at every use)
    }
  };
  set_negmb();
  float l_run = 0.f;   // this lane's share of the running sum of exponentials
  const int first_tok_wave = (int)fast_div((uint32_t)(row0 + wave * 32), p.group_div);

  // K fragment of QK step `step` = kk * 2 + a (keys 32a..32a+31, head dims 16kk..16kk+15) and
  // V^T fragment (key step kc, head dims 32dt..32dt+31), from tile buffers at LDS byte offsets
  auto read_k = [&](uint32_t kofs, int step) __attribute__((always_inline)) {
    const int a = step & 1, kk = step >> 1;
    return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(
        smem + (k_rd[kk] + kofs) + a * 32 * G::ROWB);
  };
  auto read_v = [&](uint32_t vofs, int kc, int dt) __attribute__((always_inline)) {
    typedef __attribute__((address_space(3))) s16x4_t lds_s16x4;
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4 *)(smem + (v_rd[dt] + vofs) + kc * 16 * G::ROWB));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4 *)(smem + (v_rd[dt] + vofs) + (kc * 16 + 8) * G::ROWB));
    const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, both);
  };
  // The MFMA block of one tile: O^T += V^T P^T from the V tile at vofs, then (if there is a next
  // tile) S'^T = K Q'^T - reference from the K tile at kofs: sacc[a] is keys 32a..32a+31 x this
  // wave's 32 queries, already the base-2 exponent.  The block is one stream of NS steps, one
  // MFMA each (PV: 16-key step kc x 32-dim slab dt; QK: 16-dim step kk x key half a), and the
  // fragment of step s + W - 1 is requested right before the MFMA of step s: a rolling window of
  // W fragments that keeps W - 1 MFMAs between every LDS read and its use.  The window is primed
  // (preload) before the barrier that starts the block, so the block opens with an MFMA.
  constexpr int NPV = 4 * G::DT;
  constexpr int NQK = 2 * G::KCH;
  constexpr int NS = NPV + NQK;
#ifndef BA_WIN128
#define BA_WIN128 5
#endif
  constexpr int W = D == 128 ? BA_WIN128 : 8;
  static_assert(W - 1 <= NPV, "the window is primed with V fragments only");
  auto frag_read = [&](int st, uint32_t vofs, uint32_t kofs) __attribute__((always_inline)) {
    return st < NPV ? read_v(vofs, st / G::DT, st % G::DT) : read_k(kofs, st - NPV);
  };
  auto preload = [&](uint32_t vofs, bf16x8_t (&fr)[W]) __attribute__((always_inline)) {
#pragma unroll
    for (int st = 0; st < W - 1; ++st) fr[st] = frag_read(st, vofs, 0);
  };
  // (the K fragments are requested whether or not a next tile exists: the buffer is inside LDS
  // either way and without a next tile nothing consumes them)
  // The block holds nothing but the MFMAs, their fragment reads and the waits between them: a wave
  // issues an instruction every few cycles at best, an MFMA of this shape leaves room for about three
  // others before the next one is due, and every instruction beyond that (tile copies, address
  // arithmetic, the moves that build an accumulator's start value) leaves the matrix pipe idle.
  auto mfma_block = [&](uint32_t vofs, uint32_t kofs, bool more, const bf16x8_t (&pf)[4], f32x16_t (&sacc)[2],
                        bf16x8_t (&fr)[W]) __attribute__((always_inline)) {
    // the wave in its MFMA block goes first at the issue arbiter; the other wave of the SIMD, in its
    // exponentials, fills the slots between
    __builtin_amdgcn_s_setprio(3);
#pragma unroll
    for (int st = 0; st < NPV; ++st) {
      if (st + W - 1 < NS) fr[(st + W - 1) % W] = frag_read(st + W - 1, vofs, kofs);
      const int kc = st / G::DT, dt = st % G::DT;
      oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st % W], pf[kc], oacc[dt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (more) {
#pragma unroll
      for (int st = NPV; st < NS; ++st) {
        if (st + W - 1 < NS) fr[(st + W - 1) % W] = frag_read(st + W - 1, vofs, kofs);
        const int q = st - NPV, a = q & 1, kk = q >> 1;
        if (kk == 0) {
          // the accumulator starts at minus the row's reference: the MFMA result is the exponent
          f32x16_t start;
          if constexpr (kKeepNegmb) {
            start = negmb;
          } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) start[v] = -mb;
          }
          sacc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st % W], qf[kk], start, 0, 0, 0);
        } else {
          sacc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[st % W], qf[kk], sacc[a], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };
  // QK of the very first tile (nothing to overlap it with; the reference is still 0)
  auto qk_first = [&](uint32_t kofs, f32x16_t (&sacc)[2]) __attribute__((always_inline)) {
    bf16x8_t fr[W];
#pragma unroll
    for (int q = 0; q < W - 1; ++q) fr[q] = read_k(kofs, q);
#pragma unroll
    for (int q = 0; q < NQK; ++q) {
      if (q + W - 1 < NQK) fr[(q + W - 1) % W] = read_k(kofs, q + W - 1);
      const int a = q & 1, kk = q >> 1;
      f32x16_t zero;
#pragma unroll
      for (int v = 0; v < 16; ++v) zero[v] = 0.f;
      sacc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[q % W], qf[kk], kk == 0 ? zero : sacc[a], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Row maxima of a score tile.
  auto row_max = [&](const f32x16_t (&sacc)[2]) __attribute__((always_inline)) {
    float m0 = sacc[0][0];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) m0 = fmaxf(m0, sacc[a][v]);
    return fmaxf(m0, other_half(m0));
  };
  // Move the reference by `shift`: exponents, running sum and output accumulators are all
  // re-expressed relative to the new reference.
  auto rebase = [&](f32x16_t (&sacc)[2], float shift) __attribute__((always_inline)) {
    const float alpha = __builtin_amdgcn_exp2f(-shift);
    mb += shift;
    set_negmb();
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
  // P = 2^S' rounded to bf16 (the B operand of PV); returns this lane's fp32 sum of the
  // exponentials.  (Plain adds on purpose: v_dot2c_f32_bf16 would add a packed pair in one
  // instruction, but it executes on the matrix pipe and slows to a crawl next to the other
  // wave's MFMAs.)
  auto exponentials = [&](const f32x16_t (&sacc)[2], bf16x8_t (&pf)[4]) __attribute__((always_inline)) {
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
  auto softmax = [&](const Cursor &cm, bool first, f32x16_t (&sacc)[2], bf16x8_t (&pf)[4]) __attribute__((always_inline)) {
    const bool isctx = cm.seg < n_ctx_segs;
    const int key0 = cm.ts * kTileKeys;
    const int valid = min(kTileKeys, cm.len - key0);
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
      // the first tile sets the reference: its row maximum whatever the sign (nothing visible
      // yet: stay at 0), so a row's largest exponential so far is exactly 1
      asm volatile("" ::: "memory");
      const float mx = row_max(sacc);
      const float shift = mx == -INFINITY ? 0.f : mx;
      mb = shift;
      set_negmb();
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[a][v] -= shift;
    }
    float tsum = exponentials(sacc, pf);
    if (__builtin_amdgcn_ballot_w64(!(tsum < kRebaseAbove)) != 0) {  // overflow guard: practically never
      asm volatile("" ::: "memory");
      rebase(sacc, fmaxf(row_max(sacc), 0.f));  // only ever raise the reference here
      tsum = exponentials(sacc, pf);
    }
    l_run += tsum;
  };
  // ---- the walk over the key tiles ------------------------------------------------------------------
  // Tile i (counted from t_begin) has its K in K buffer i % 4 and its V in V buffer i % 4.  Every wave
  // runs the same chain  softmax(i), PV(i), QK(i+1)  but the two waves of a SIMD (w and w + 4) run
  // it half a period apart: time is cut into half-periods that end in a workgroup barrier, and in
  // each of them one wave of a SIMD is in its exponentials (VALU) while the other is in its MFMA
  // block, so that neither unit waits for the other.
  //     half-period   -1      0        1            2            3         ...
  //     waves 0..3   QK(0)  SM(0)  PV(0) QK(1)    SM(1)      PV(1) QK(2)
  //     waves 4..7     -    QK(0)    SM(0)     PV(0) QK(1)     SM(1)
  // Waves 0..3 fetch K(i+3) and waves 4..7 V(i+3) in the softmax half of iteration i; at
  // the end of that half a wave waits until the tile it started two iterations earlier
  // (K(i+1) resp. V(i+1)) has landed, and the barrier that ends the half-period publishes it.  A
  // buffer is refilled only after the barrier that follows its last reader.
  Cursor cp = cursor_at(t_begin);  // the next tile to copy
  const char *cp_ptr = nullptr;    // where the tile after the last copied one starts (same segment)
  auto first_copy = [&](int j) __attribute__((always_inline)) {  // tile j = 0, 1, 2 of the walk, before the loop
    if (j < n_t) {
      // (as in the loop: a full tile that follows the last copied one in memory needs the pointer only)
      const uint32_t rb = cp.seg >= n_ctx_segs ? f_rb : c_rb;
      if (j > 0 && cp.ts > 0 && rb == prim_rb && (cp.ts + 1) * kTileKeys <= cp.len) {
        const uint32_t dst = lds_copy + (uint32_t)j * TB;
#pragma unroll
        for (int i = 0; i < G::IPW; ++i) lds_dma16(cp_ptr, g_src[i], dst + i * 1024);
        cp_ptr += (uint64_t)(prim_rb * (uint32_t)kTileKeys);
      } else {
        const CopyJob c = copy_prepare(cp, j);
#pragma unroll
        for (int i = 0; i < G::IPW; ++i) copy_part(c, i);
        cp_ptr = c.ptr + (uint64_t)(c.rb * (uint32_t)kTileKeys);
      }
      advance(cp);
    }
  };
  // Start-up order.  Every workgroup of a launch starts at the same moment and would ask for its
  // first three tiles of either kind and its query rows at once: 160 KB per compute unit, which its
  // vector-memory path takes some 2,500 cycles to move, and the first MFMA waited for all of it.  The
  // first scores need tile 0 and the query rows only: those are asked for first and waited for; tiles
  // 1 and 2 are asked for behind the barrier that publishes tile 0 and arrive while the first scores
  // and the first exponentials are worked out (the loop's own waits cover them, as every later tile).
  first_copy(0);
  probe_mark(3);  // tile 0 is on its way

  // ---- Q fragments (B operand of S^T = K Q^T).  With rotary embedding the rows come from the
  //      RoPE pre-pass, already rotated and multiplied by scale * log2(e); otherwise they are the
  //      caller's and are scaled here, before one rounding back to bf16.  With a block table the
  //      cached keys of block b stay at the positions they were encoded at and the queries are
  //      turned back by the block's shift instead (rot >= 0: row of the table of rotations), which
  //      gives the same scores as re-encoding the keys (Eq. 2 and 3 applied to q instead of k) ------
  // With a block table the walk keeps more scalars alive than the register file holds (two cursors
  // over the table on top of everything the epilogue needs), and what does not fit is parked in
  // lanes of a vector register and fetched back on every iteration.  The rare parts of that
  // kernel (this reload, the epilogue) therefore read their kernel arguments again from the
  // argument segment (`p` is its first member) through a pointer the compiler cannot see through.
  typedef const __attribute__((address_space(4))) AttnParams *KParams;
  auto args_again = [&]() __attribute__((always_inline)) {
    KParams kp = (KParams)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(kp));
    return kp;
  };
#define BA_ARG(field) (kBlocks ? kp->field : p.field)
  // this lane's query row: where its fragments start, and its token inside the problem
  struct QRow {
    const uint16_t *ptr;
    int tok;
  };
  auto q_row = [&]() __attribute__((always_inline)) {
    KParams kp = kBlocks ? args_again() : nullptr;
    const FastDiv gdiv = {BA_ARG(group_div.mul), BA_ARG(group_div.sh1), BA_ARG(group_div.sh2)};
    // (addresses are rebuilt from the row number each time: with a block table this runs inside the
    // loop, and hoisted address registers would not fit next to the accumulators)
    int row_v = my_row;
    asm volatile("" : "+v"(row_v));
    QRow r;
    r.tok = (int)fast_div((uint32_t)row_v, gdiv);
    const int g = row_v - r.tok * Gq;
    const int head = kvh * Gq + g;
    r.ptr = BA_ARG(q) + (int64_t)(pr.q_tok0 + r.tok) * BA_ARG(q_st) + (int64_t)head * BA_ARG(q_sh) + hf * 8;
    return r;
  };
  // fragments as loaded -> rotated / scaled as the call asks -> qf
  auto q_finish = [&](u32x4_t (&raw)[G::KCH], int tok_v, int rot) __attribute__((always_inline)) {
    KParams kp = kBlocks ? args_again() : nullptr;
    // rotate the fragments by the angles of a table row: entry j = (cos, sin) (times a scale, if any)
    auto rotate_by = [&](const f32x4_t *tab) __attribute__((always_inline)) {
      if (BA_ARG(rope_layout) == 0) {
#pragma unroll
        for (int kk = 0; kk < G::KCH; ++kk) {
          // this lane's pairs: frequencies kk * 8 + hf * 4 + e
          const f32x4_t cs0 = tab[(kk * 8 + hf * 4) / 2], cs1 = tab[(kk * 8 + hf * 4) / 2 + 1];
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
          // dims kk * 16 + hf * 8 + (0..7) pair with the same dims + D/2: frequencies = those dims
          f32x4_t cs[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) cs[u] = tab[(kk * 16 + hf * 8) / 2 + u];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float c0 = cs[e][0], s0 = cs[e][1], c1 = cs[e][2], s1 = cs[e][3];
            const uint32_t wa = raw[kk][e], wb = raw[kk + G::KCH / 2][e];
            const float xa0 = bf16_lo(wa), xa1 = bf16_hi(wa), xb0 = bf16_lo(wb), xb1 = bf16_hi(wb);
            raw[kk][e] = pack_bf16(c0 * xa0 - s0 * xb0, c1 * xa1 - s1 * xb1);
            raw[kk + G::KCH / 2][e] = pack_bf16(s0 * xa0 + c0 * xb0, s1 * xa1 + c1 * xb1);
          }
        }
      }
    };
    if (!BA_ARG(q_ready)) {
      if (BA_ARG(q_table)) {
        // un-rotated rows and the pre-pass's table of scale * (cos, sin) per token: rotate here, so that
        // the rotated queries never make a round trip through memory
        // (lanes beyond the problem's rows hold zeros: any row of the table will do, take an existing one)
        rotate_by(reinterpret_cast<const f32x4_t *>(
            BA_ARG(q_table) + (int64_t)((BA_ARG(q_table_by_pos) ? 0 : pr.q_tok0) + (row_ok ? tok_v : 0)) * D));
      } else {
#pragma unroll
        for (int kk = 0; kk < G::KCH; ++kk)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            raw[kk][e] = pack_bf16(bf16_lo(raw[kk][e]) * BA_ARG(scale_log2e), bf16_hi(raw[kk][e]) * BA_ARG(scale_log2e));
      }
    }
    if (kBlocks && rot >= 0) {
      // (cos, sin) of minus the block's shift times theta_j, j = 0 .. D/2 - 1
      rotate_by(reinterpret_cast<const f32x4_t *>(BA_ARG(blk_rot) + (int64_t)rot * D));
    }
    // (the empty asm makes the compiler wait for these loads HERE: left pending, it would wait for
    // them at the first use of the fragments inside the loop's MFMA block, on every iteration, and
    // that wait also covers the tile copies just started there)
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) {
      asm volatile("" : "+v"(raw[kk]));
      qf[kk] = __builtin_bit_cast(bf16x8_t, raw[kk]);
    }
  };
  auto load_q = [&](int rot) __attribute__((always_inline)) {
    const QRow r = q_row();
    u32x4_t raw[G::KCH];
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) {
      u32x4_t z = {0u, 0u, 0u, 0u};
      raw[kk] = row_ok ? *reinterpret_cast<const u32x4_t *>(r.ptr + kk * 16) : z;
    }
    q_finish(raw, r.tok, rot);
  };
  // The first load of the query rows, before the loop.  A lane fetching the sixteen-byte pieces of its
  // own row touches a cache line per lane and instruction (thirty-two lines for one kilobyte), and a
  // workgroup's 64 KB of query rows then take some 2.5 microseconds to arrive, five times as long as
  // its first tiles.  Here the rows are fetched whole instead (LDS-direct, four 256-byte rows per
  // wave instruction) into a slice of tile buffers 1 and 2 of the wave's kind, which are idle until
  // the first barrier, laid out as a K tile of 32 rows; the fragments are then read from the slice
  // at the offsets of a K fragment.  Each wave reads only what it fetched itself: no barrier.
  auto load_q_first = [&](int rot) __attribute__((always_inline)) {
    KParams kp = kBlocks ? args_again() : nullptr;
    const FastDiv gdiv = {BA_ARG(group_div.mul), BA_ARG(group_div.sh1), BA_ARG(group_div.sh2)};
    const uint32_t slice = (role_b ? VBASE : 0u) + TB + (uint32_t)(wave & (kWaves / 2 - 1)) * (32 * G::ROWB);
    static_assert((kWaves / 2) * 32 * G::ROWB == 2 * TB, "the slices of a kind's four waves fill its tile buffers 1 and 2");
    const int wave_row0 = row0 + wave * 32;
    const int tok_first = (int)fast_div((uint32_t)min(wave_row0, n_rows - 1), gdiv);  // wave-uniform
    const char *qbase = (const char *)(BA_ARG(q) + (int64_t)(pr.q_tok0 + tok_first) * BA_ARG(q_st) +
                                       (int64_t)(kvh * Gq) * BA_ARG(q_sh));
    const uint32_t st_b = (uint32_t)BA_ARG(q_st) * 2u, sh_b = (uint32_t)BA_ARG(q_sh) * 2u;  // (the host checked that they fit)
#pragma unroll
    for (int j = 0; j < 32 / G::RPI; ++j) {
      const int r_in = j * G::RPI + lane / G::CPR, pos = lane % G::CPR;
      const int r = min(wave_row0 + r_in, n_rows - 1);  // rows beyond the problem: its last row, zeroed below
      const int tok = (int)fast_div((uint32_t)r, gdiv);
      const uint32_t off = (uint32_t)(tok - tok_first) * st_b + (uint32_t)(r - tok * Gq) * sh_b +
                           ((uint32_t)(pos ^ ((r_in / G::LPR) & (G::CPR - 1))) << 4);
      lds_dma16(qbase, off, (uint32_t)(uintptr_t)smem + slice + j * 1024);
    }
    dma_wait<0>();  // tile 0 (this wave's share) and the query rows are complete from here on
    u32x4_t raw[G::KCH];
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) {
      raw[kk] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t *>(smem + slice + k_rd[kk]);
      if (!row_ok) raw[kk] = u32x4_t{0u, 0u, 0u, 0u};
    }
    q_finish(raw, my_tok, rot);
  };
  Cursor cm = cursor_at(t_begin);  // the tile whose softmax comes next
  auto rot_of = [&](int sg) __attribute__((always_inline)) {
    if constexpr (kBlocks) return sg < n_ctx_segs ? meta.rot_base + pr.blk0 + sg : -1;
    return -1;
  };
  if (p.q_rows_fit32) {
    load_q_first(rot_of(cm.seg));
  } else {
    load_q(rot_of(cm.seg));
    dma_wait<0>();
  }
  probe_mark(6);
  f32x16_t sacc[2];
  bf16x8_t pf[4];
  bf16x8_t fr[W];
  if (n_t > 0) {
    if (!role_b) {
      wg_barrier();  // tile 0 of both kinds is visible
      first_copy(1);
      first_copy(2);
      if (wave_has_rows) qk_first(0, sacc);
      wg_barrier();
    } else {
      wg_barrier();
      first_copy(1);
      first_copy(2);
      wg_barrier();
      if (wave_has_rows) qk_first(0, sacc);
      wg_barrier();
    }
    // One iteration.  The copy of tile i+3 is prepared here, in the softmax half, where scalar
    // instructions cost nothing on the matrix pipe: a full tile that follows the last copied one in
    // memory only needs the pointer carried along; anything else (first tile of a segment, ragged
    // tile, other stride) is worked out from the cursor.  `steady` (compile time) promises the
    // common case: tiles i+1 and i+3 exist, tile i+1 lies in the same segment as tile i, and the
    // copy is such a following full tile.
    probe_mark(7);  // (wave 0:) the first scores are done, the loop begins
    const uint64_t tile_bytes = (uint64_t)(prim_rb * (uint32_t)kTileKeys);
    auto iteration = [&](auto steady_c, int i) __attribute__((always_inline)) {
      constexpr bool steady = decltype(steady_c)::value;
      if (wave_has_rows) softmax(cm, i == 0, sacc, pf);
      // Tile i+1 opens a segment of a block table: new query fragments.  Waves 0..3 turn theirs here;
      // waves 4..7 have done so right behind their previous MFMA block (see below), in the same
      // half-period, so that the workgroup stalls once per boundary, not twice.
      if (kBlocks && !steady && i + 1 < n_t && cm.rem == 1 && (!role_b || i == 0)) {
        __builtin_amdgcn_s_setprio(3);
        load_q(rot_of(cm.seg + 1));
        __builtin_amdgcn_s_setprio(0);
      }
      // This wave's share of the copy of tile i+3 goes out here, in the softmax half, where the wave
      // has issue slots to spare (its buffer's last readers finished before the barrier that opened
      // this half-period: K(i-1) was last read by QK(i-1), V(i-1) by PV(i-1), both in MFMA blocks
      // that ended at or before that barrier for every wave).
      const bool copy = steady || i + 3 < n_t;
      if (copy) {
        CopyJob cj;
        cj.ptr = cp_ptr;
        cj.dst = lds_copy + (uint32_t)((i + 3) & (kNumKBuf - 1)) * TB;
        cj.rb = prim_rb;
        cj.valid = kTileKeys;
        cj.full = true;
        uint32_t cp_off[G::IPW];
#pragma unroll
        for (int u = 0; u < G::IPW; ++u) cp_off[u] = g_src[u];
        const uint32_t rb = cp.seg >= n_ctx_segs ? f_rb : c_rb;
        if (steady || (cp.ts > 0 && rb == prim_rb && (cp.ts + 1) * kTileKeys <= cp.len)) {
          cp_ptr += tile_bytes;
        } else {
          asm volatile("" ::: "memory");
          cj = copy_prepare(cp, (i + 3) & (kNumKBuf - 1));
          if (!cj.full) {
#pragma unroll
            for (int u = 0; u < G::IPW; ++u)
              cp_off[u] = (uint32_t)min(copy_row(u), cj.valid - 1) * cj.rb + copy_chunk(u);
          }
          cp_ptr = cj.ptr + (uint64_t)(cj.rb * (uint32_t)kTileKeys);
        }
        advance(cp);
#pragma unroll
        for (int u = 0; u < G::IPW; ++u) lds_dma16(cj.ptr, cp_off[u], cj.dst + u * 1024);
      }
      // tile i+1 of this wave's kind must have landed before the barrier; the copies that may be
      // younger are tile i+2's and the one just started
      if (steady || copy) dma_wait<2 * G::IPW>();
      else if (i + 2 < n_t) dma_wait<G::IPW>();
      else dma_wait<0>();
      const uint32_t vofs = VBASE + (i & (kNumVBuf - 1)) * TB;
      if (wave_has_rows) preload(vofs, fr);
      wg_barrier();
      if (wave_has_rows) mfma_block(vofs, ((i + 1) & (kNumKBuf - 1)) * TB, steady || i + 1 < n_t, pf, sacc, fr);
      if constexpr (kBlocks && !steady) {
        advance(cm);
        if (role_b && i + 2 < n_t && cm.rem == 1) {  // (QK of tile i+1 is done: the fragments are free)
          __builtin_amdgcn_s_setprio(3);
          load_q(rot_of(cm.seg + 1));
          __builtin_amdgcn_s_setprio(0);
        }
        if (!role_b || i + 1 < n_t) wg_barrier();
      } else {
        if (steady || !role_b || i + 1 < n_t) wg_barrier();
        advance(cm);
      }
    };
    // With a contiguous context (or none) the steady iterations form one run from the start: until
    // the copy cursor or the compute cursor reaches the end of the segment they start in.
    int n_steady = 0;
    if (!kBlocks) {
      const int full_tiles = cp.len / kTileKeys;  // of the segment the copy cursor is in
      const bool fast = (cp.seg >= n_ctx_segs ? f_rb : c_rb) == prim_rb && cp.ts > 0;
      n_steady = fast ? max(0, min(min(n_t - 3, full_tiles - cp.ts), cm.rem - 1)) : 0;
    }
    int i = 0;
#pragma unroll 1
    for (; i < n_steady; ++i) iteration(std::true_type{}, i);
#pragma unroll 1
    for (; i < n_t; ++i) iteration(std::false_type{}, i);
  }
  static_assert(kNumKBuf == 4 && kNumVBuf == 4, "the copy distances above assume four buffers of each kind");
  if (kProbe && p.wg_clock && threadIdx.x == 0) {
    unsigned long long *rec = p.wg_clock + (size_t)blockIdx.x * kProbeRecord;
    rec[4] = (unsigned long long)clock64();
    rec[5] = (unsigned long long)wall_clock64();
  }

  // ---- epilogue -----------------------------------------------------------------------------------
  KParams kp = kBlocks ? args_again() : nullptr;
  const float l_tot = l_run + other_half(l_run);
  // Every piece is normalised by its own sum (a convex combination of v rows, so it fits fp16 when
  // it is a split partial); a piece that saw no key is all zeros.
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  if (BA_ARG(n_splits) > 1) {
    // A split partial leaves in the layout the accumulators have: lane (col, hf) holds, of query row
    // `col`, the head dims 32 dt + 8 q4 + 4 hf + (0..3); store k = 2 dt + q4 / 2 carries two such
    // groups of four (q4 even, q4 odd) as eight fp16, and the wave's 64 lanes write 1 KB of consecutive
    // memory per store.  No transposition, no per-row addresses: the merge kernel undoes the layout.
    const int64_t unit = ((int64_t)(BA_ARG(tile_base) + rowtile) * BA_ARG(n_kv_heads) + kvh) * kWaves + wave;
    const int64_t slot = (int64_t)split * BA_ARG(part_units) + unit;
    char *dst = (char *)BA_ARG(part_o) + slot * (int64_t)(32 * D * 2) + lane * 16;
#pragma unroll
    for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
      for (int qp = 0; qp < 2; ++qp) {
        u32x4_t w;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int v0 = (qp * 2 + u) * 4;
          w[u * 2] = pack_f16(oacc[dt][v0] * inv, oacc[dt][v0 + 1] * inv);
          w[u * 2 + 1] = pack_f16(oacc[dt][v0 + 2] * inv, oacc[dt][v0 + 3] * inv);
        }
        *reinterpret_cast<u32x4_t *>(dst + (dt * 2 + qp) * 1024) = w;
      }
    if (hf == 0) {
      float2 ml = {l_tot > 0.f ? mb : -INFINITY, l_tot};  // reference in log2 units; -inf: nothing visible
      *reinterpret_cast<float2 *>(BA_ARG(part_ml) + (slot * 32 + col) * 2) = ml;
      if (split == 0) {
        // (the row's token is worked out again, from a copy of the row number the compiler cannot
        // see through: kept from before the walk it would be spilled)
        int row_e = my_row;
        asm volatile("" : "+v"(row_e));
        const FastDiv gd = {BA_ARG(group_div.mul), BA_ARG(group_div.sh1), BA_ARG(group_div.sh2)};
        const int tok_e = (int)fast_div((uint32_t)row_e, gd);
        const int g = row_e - tok_e * Gq;
        BA_ARG(part_idx)[unit * 32 + col] = row_e < n_rows ? (pr.q_tok0 + tok_e) * BA_ARG(n_q_heads) + kvh * Gq + g : -1;
      }
    }
    if (kProbe && p.wg_clock && threadIdx.x == 0) {
      probe_mark(8);                    // the partial's stores are issued
      __builtin_amdgcn_s_waitcnt(0);
      probe_mark(9);                    // and complete
    }
    return;
  }
  // One piece (no splits): each wave transposes its O^T through its own slice of LDS, half of the head
  // dimension at a time, so that rows leave as contiguous lines.  The slices lie in the K buffers,
  // and every wave's last K read precedes the last barrier the other waves passed; waves 4..7 may
  // still be reading their last V tile, which lies elsewhere.
  const FastDiv gdiv_e = {BA_ARG(group_div.mul), BA_ARG(group_div.sh1), BA_ARG(group_div.sh2)};
  constexpr int HD = D / 2;               // floats per staged row piece
  constexpr int HCH = HD / 4;             // 16-byte chunks per piece (16 or 8)
  constexpr int PITCH = HD * 4;           // bytes per staged row piece (256 or 128)
  constexpr int HLPR = 256 / PITCH;       // pieces per 256-byte LDS line
  lds_char *stage = smem + wave * (32 * PITCH);
  // (the swizzled chunk offsets below are the same expressions as the K fragment offsets of the loop:
  // computed from an opaque copy of the lane's column, or the compiler keeps them alive across the
  // whole walk, where there is no register for them, and spills them)
  int col_e = col;
  asm volatile("" : "+v"(col_e));
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
            stage + col_e * PITCH + ((chunk ^ ((col_e / HLPR) & (HCH - 1))) << 4)) = w;
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
        const int i = (int)fast_div((uint32_t)r, gdiv_e);
        const int g = r - i * Gq;
        const int head = kvh * Gq + g;
        const int d = half * HD + ch * 4;
        uint2 o2;
        o2.x = pack_bf16(w[0], w[1]);
        o2.y = pack_bf16(w[2], w[3]);
        *reinterpret_cast<uint2 *>(BA_ARG(o) + (int64_t)(pr.q_tok0 + i) * BA_ARG(o_st) + (int64_t)head * BA_ARG(o_sh) + d) = o2;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

#undef BA_ARG

// Merge split partials in split order.  Split i holds its own normalised output o_i (fp16), its
// reference m_i (log2 units; -inf if it saw no key) and its sum l_i:
//   m = max m_i,  w_i = 2^(m_i - m) l_i,  o = sum_i w_i o_i / sum_i w_i.
// The partials lie as the attention kernel's accumulators held them (AttnParams::part_o): a thread
// here is (unit, store k, lane) of that layout and owns eight output elements of one row -- head dims
// 32 (k / 2) + 16 (k & 1) + 4 hf + (0..3) and the same + 8 -- so every load is 16 bytes and a wave
// reads 1 KB of consecutive memory per split.  SG = 1: a thread merges all splits one after the
// other.  SG = 4 (many splits, few rows): four groups of threads take every fourth split each, so that
// all loads of a row are in flight at once, and the groups' sums are merged through LDS, group 0 first.
template <int D, int SG>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(AttnParams p) {
  constexpr int K = D / 16;                          // 16-byte stores per lane of the layout
  constexpr int KPB = kCombineThreads / (64 * SG);   // layout stores (k values) per workgroup
  static_assert(KPB >= 1 && K % KPB == 0, "a workgroup covers whole k values of one unit");
  constexpr int BPU = K / KPB;                       // workgroups per unit
  const int g = threadIdx.x / (64 * KPB);            // which group of splits
  const int kl = (threadIdx.x / 64) % KPB;
  const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
  const int64_t unit = blockIdx.x / BPU;
  const int k = (int)(blockIdx.x % BPU) * KPB + kl;
  // all loads are unconditional and independent, so they go out together
  constexpr int MAXS = 32;  // the host never asks for more splits
  const int n_mine = (p.n_splits - g + SG - 1) / SG;  // splits g, g + SG, ...
  const float2 *ml = reinterpret_cast<const float2 *>(p.part_ml) + unit * 32 + col;
  const char *po = (const char *)p.part_o + unit * (int64_t)(32 * D * 2) + k * 1024 + lane * 16;
  const int64_t ml_stride = p.part_units * 32, o_stride = p.part_units * (int64_t)(32 * D * 2);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float l = 0.f, m = -INFINITY;
  if (n_mine <= 8) {
    // the common case (up to eight splits per thread): every load of the thread is requested before
    // anything is used, a split beyond the thread's last reads its last one again with weight zero
    float2 mls[8];
    u32x4_t os[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int s = g + min(j, n_mine - 1) * SG;
      mls[j] = ml[s * ml_stride];
      os[j] = *reinterpret_cast<const u32x4_t *>(po + s * o_stride);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < n_mine) m = fmaxf(m, mls[j].x);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float w = (j >= n_mine || mls[j].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mls[j].x - m) * mls[j].y;
      l += w;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += w * f16_lo(os[j][i]);
        acc[2 * i + 1] += w * f16_hi(os[j][i]);
      }
    }
  } else {
    float wgt[MAXS];
#pragma unroll 8
    for (int j = 0; j < n_mine; ++j) {
      const int s = g + j * SG;
      wgt[j & (MAXS - 1)] = ml[s * ml_stride].x;
      m = fmaxf(m, wgt[j & (MAXS - 1)]);
    }
#pragma unroll 8
    for (int j = 0; j < n_mine; ++j) {
      const int s = g + j * SG;
      const float ms = wgt[j & (MAXS - 1)];
      const float ls = ml[s * ml_stride].y;
      const float w = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - m) * ls;
      const u32x4_t o = *reinterpret_cast<const u32x4_t *>(po + s * o_stride);
      l += w;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += w * f16_lo(o[i]);
        acc[2 * i + 1] += w * f16_hi(o[i]);
      }
    }
  }
  const int idx = p.part_idx[unit * 32 + col];
  if constexpr (SG > 1) {
    // (reference, sum, eight partial outputs) of every thread; group 0 merges them in group order
    __shared__ float part[SG][64 * KPB][10 + 1];
    float *mine = part[g][threadIdx.x % (64 * KPB)];
    mine[0] = m;
    mine[1] = l;
#pragma unroll
    for (int i = 0; i < 8; ++i) mine[2 + i] = acc[i];
    __syncthreads();
    if (g != 0) return;
    float mm = m;
#pragma unroll
    for (int h = 1; h < SG; ++h) mm = fmaxf(mm, part[h][threadIdx.x][0]);
    const float w0 = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mm);
    l *= w0;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] *= w0;
#pragma unroll
    for (int h = 1; h < SG; ++h) {
      const float *o = part[h][threadIdx.x];
      const float wh = (o[0] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(o[0] - mm);
      l += wh * o[1];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += wh * o[2 + i];
    }
  }
  if (idx < 0) return;  // a row beyond the problem's last
  const float inv = 1.0f / l;
  const int tokn = idx / p.n_q_heads;
  const int head = idx - tokn * p.n_q_heads;
  const int d = 32 * (k >> 1) + 16 * (k & 1) + 4 * hf;
  uint16_t *orow = p.o + (int64_t)tokn * p.o_st + (int64_t)head * p.o_sh + d;
  uint2 lo, hi;
  lo.x = pack_bf16(acc[0] * inv, acc[1] * inv);
  lo.y = pack_bf16(acc[2] * inv, acc[3] * inv);
  hi.x = pack_bf16(acc[4] * inv, acc[5] * inv);
  hi.y = pack_bf16(acc[6] * inv, acc[7] * inv);
  *reinterpret_cast<uint2 *>(orow) = lo;
  *reinterpret_cast<uint2 *>(orow + 8) = hi;
}

template <int D, typename Meta>
hipError_t launch_attn_t(const AttnParams &p, const Meta &meta, hipStream_t stream) {
  const int64_t n_wg = (int64_t)p.total_tiles * p.n_kv_heads * p.n_splits;
  if (n_wg == 0) return hipSuccess;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  constexpr size_t lds = Geo<D>::LDS;
  static_assert((size_t)kWaves * 32 * D * 2 <= lds, "epilogue staging must fit the tile buffers");
  static_assert(lds <= 160 * 1024, "gfx950 has 160 KB of LDS per workgroup");
  // more than 64 KB of dynamic LDS has to be asked for once per kernel (setting it twice, from two
  // host threads at once, is harmless)
  static std::atomic<bool> raised{false};
  if (lds > 64 * 1024 && !raised.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_kernel<D, Meta>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    raised.store(true, std::memory_order_release);
  }
  AttnParams pl = p;  // with the launch's divisors
  pl.tiles_div = make_fast_div((uint32_t)p.total_tiles);
  pl.kv_group = p.kv_group > 0 ? p.kv_group : kDefaultKvGroup;  // (the planner's choice, or the default)
  // (likewise the XCDs' runs; anything that is not a permutation fit for this launch reads as "in order")
  pl.xcd_runs = p.xcd_runs != 0 && xcd_runs_valid(p.xcd_runs, (unsigned)n_wg) ? p.xcd_runs : kIdentityXcdRuns;
  pl.item_divs = make_item_divs(ItemOrder{p.total_tiles, p.n_kv_heads, p.n_splits, pl.kv_group});
  pl.split_divs = make_split_divs(p.n_splits);
  pl.q_rows_fit32 = p.q_st > 0 && p.q_sh > 0 && 32 * p.q_st * 2 + (int64_t)p.group * p.q_sh * 2 < (int64_t)1 << 32;
  hipLaunchKernelGGL((attn_kernel<D, Meta>), dim3((unsigned)n_wg), dim3(kThreads), lds, stream, pl, meta);
  return hipGetLastError();
}

}  // namespace


hipError_t launch_attn_encode(const AttnParams &p, const EncodeMeta &meta, hipStream_t stream) {
  if (p.head_dim == 128) return launch_attn_t<128, EncodeMeta>(p, meta, stream);
  if (p.head_dim == 64) return launch_attn_t<64, EncodeMeta>(p, meta, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_attn_final(const AttnParams &p, const FinalMeta &meta, hipStream_t stream) {
  if (p.head_dim == 128) return launch_attn_t<128, FinalMeta>(p, meta, stream);
  if (p.head_dim == 64) return launch_attn_t<64, FinalMeta>(p, meta, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_attn_final_blocks(const AttnParams &p, const FinalBlocksMeta &meta, hipStream_t stream) {
  if (p.head_dim == 128) return launch_attn_t<128, FinalBlocksMeta>(p, meta, stream);
  if (p.head_dim == 64) return launch_attn_t<64, FinalBlocksMeta>(p, meta, stream);
  return hipErrorInvalidValue;
}
hipError_t launch_attn_final_blocks(const AttnParams &p, const FinalBlocksMetaSmall &meta, hipStream_t stream) {
  if (p.head_dim == 128) return launch_attn_t<128, FinalBlocksMetaSmall>(p, meta, stream);
  if (p.head_dim == 64) return launch_attn_t<64, FinalBlocksMetaSmall>(p, meta, stream);
  return hipErrorInvalidValue;
}

template <int D, int SG>
void launch_combine_t(const AttnParams &p, hipStream_t stream) {
  constexpr int BPU = (D / 16) / (kCombineThreads / (64 * SG));  // workgroups per unit
  hipLaunchKernelGGL((combine_kernel<D, SG>), dim3((unsigned)(p.part_units * BPU)), dim3(kCombineThreads), 0, stream, p);
}

hipError_t launch_combine(const AttnParams &p, hipStream_t stream) {
  if (p.part_units == 0) return hipSuccess;
  if (p.part_units * (p.head_dim / 16) > 0x7fffffff) return hipErrorInvalidValue;
  const bool many = p.n_splits > 8;  // more splits than one thread keeps in flight: four groups of threads per row
  if (p.head_dim == 128) {
    if (many) launch_combine_t<128, 4>(p, stream); else launch_combine_t<128, 1>(p, stream);
  } else if (p.head_dim == 64) {
    if (many) launch_combine_t<64, 4>(p, stream); else launch_combine_t<64, 1>(p, stream);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ba
