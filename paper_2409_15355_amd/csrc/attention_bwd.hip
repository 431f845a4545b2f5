// Backward pass of whole-prompt Block-attention (arXiv 2409.15355, Section 2.4: the mask a block
// fine-tune step trains under).  With P the masked softmax of S = scale * q^ k^T (q^, k^ rotated at
// their positions inside the prompt), O = P V and dO given:
//   delta_r = sum_d dO_rd O_rd,   dV = P^T dO,   dP = dO V^T,   dS = P o (dP - delta),
//   dq^ = scale * dS k^,          dk^ = scale * dS^T q^.
// Nothing of the forward pass is kept but O and the rows' log-sum-exps L: P is recomputed as
// exp(S - L).  Two kernels, so that every sum has one owner and no atomics are needed:
//   - bwd_dq_kernel: a workgroup owns 128 packed query rows (as the forward kernel for short items
//     does) and walks the key tiles its rows see; it accumulates dq^.
//   - bwd_dkv_kernel: a workgroup owns 128 keys of one block and KV head and walks the 32-row
//     query tiles that see them (the rest of its own block, and the prompt's last block if it is a
//     passage); it accumulates dk^ and dV over all query heads of the group.
// Each turns its gradient of the rotated tensor back to the un-rotated frame in its epilogue, with the
// (cos, sin) table of the RoPE pre-pass (Eq. 1 is orthogonal: the transposed map is the rotation by
// minus the angle).
//
// Operand layouts are the forward kernel's: products are computed transposed with
// v_mfma_f32_32x32x16_bf16, the owner's side along lanes and in registers as B operands, the
// walked side from LDS tiles as A operands (16-byte row reads for the products that contract over
// head_dim, LDS transpose reads for those that contract over the walked index), and a probability
// tile in accumulator layout is directly the B operand of the next product.
#include <atomic>
#include <type_traits>

#include "ba_device.h"
#include "ba_lds.h"

namespace ba {
namespace {

constexpr int kBWaves = 4;
constexpr int kBThreads = kBWaves * 64;
constexpr int kBKeys = 32;  // walked rows (keys, or packed query rows) per tile
constexpr int kBBuf = 3;    // tile buffers
constexpr int kKvRows = 32; // packed query rows per tile of the dk/dv kernel
constexpr float kLn2 = 0.6931471805599453f, kLog2e = 1.4426950408889634f;

template <int D>
struct BGeo {
  static constexpr int KCH = D / 16;
  static constexpr int DT = D / 32;
  static constexpr int CPR = D / 8;
  static constexpr int ROWB = D * 2;
  static constexpr int LPR = 256 / ROWB;
  static constexpr int TILEB = kBKeys * ROWB;
  static constexpr int RPI = 1024 / ROWB;             // rows filled by one LDS-direct wave instruction
  static constexpr int IPW = kBKeys / RPI / kBWaves;  // such instructions per wave and tile
  static constexpr int QRPI = 64 / CPR;               // whole rows per plain load instruction
  static_assert(IPW >= 1 && 32 / QRPI == KCH, "tile geometry");
};

// row `row` of a tile, 16-byte chunk `chunk`: every tile here uses the one swizzle
template <int D>
__device__ __forceinline__ uint32_t tile_ofs(int row, int chunk) {
  using G = BGeo<D>;
  return (uint32_t)(row * G::ROWB + ((chunk ^ ((row / G::LPR) & (G::CPR - 1))) << 4));
}

// A gradient in the rotated frame, held in accumulator layout (lane = row `col`, register v of slab dt =
// head dim 32 dt + (v >> 2) * 8 + hf * 4 + (v & 3)), turned back to the un-rotated frame: the
// transposed map of Eq. 1, [x', y'] = [c x + s y, -s x + c y] per pair, times `mul`.  tab = the row's
// entry of the pre-pass's table, (cos, sin) per pair times some factor that `mul` takes out again.
template <int D>
__device__ __forceinline__ void rotate_back(f32x16_t (&acc)[D / 32], const f32x4_t *tab, int hf, bool halves, float mul) {
  constexpr int DT = D / 32;
  if (!halves) {
    // pairs (d, d + 1): the four values of (dt, q4) are pairs 2 m and 2 m + 1 with m = dt * 8 + q4 * 2 + hf
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4_t t = tab[dt * 8 + q4 * 2 + hf];
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const float c = t[2 * h2] * mul, sn = t[2 * h2 + 1] * mul;
          const float x = acc[dt][q4 * 4 + 2 * h2], y = acc[dt][q4 * 4 + 2 * h2 + 1];
          acc[dt][q4 * 4 + 2 * h2] = c * x + sn * y;
          acc[dt][q4 * 4 + 2 * h2 + 1] = c * y - sn * x;
        }
      }
  } else {
    // pairs (d, d + D/2): slab dt pairs with slab dt + DT/2; the four values of (dt, q4) are pairs
    // j .. j + 3 with j = dt * 32 + q4 * 8 + hf * 4
#pragma unroll
    for (int dt = 0; dt < DT / 2; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const f32x4_t t = tab[(dt * 32 + q4 * 8 + hf * 4) / 2 + h2];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const float c = t[2 * e] * mul, sn = t[2 * e + 1] * mul;
            const float x = acc[dt][q4 * 4 + 2 * h2 + e], y = acc[dt + DT / 2][q4 * 4 + 2 * h2 + e];
            acc[dt][q4 * 4 + 2 * h2 + e] = c * x + sn * y;
            acc[dt + DT / 2][q4 * 4 + 2 * h2 + e] = c * y - sn * x;
          }
        }
  }
}

// ---------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBThreads, 2) void bwd_dq_kernel(AttnParams p, PromptMeta meta, BwdParams bp) {
  using G = BGeo<D>;
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char *smem = (lds_char *)smem_generic;
  // LDS map: buffer b = bytes [2 b TB, 2 (b + 1) TB): its K tile, then its V tile
  constexpr uint32_t TB = G::TILEB;

  uint32_t id = blockIdx.x;
  {
    constexpr uint32_t kXcds = 8;
    const uint32_t n_wg = gridDim.x, q = n_wg / kXcds, r = n_wg % kXcds, x = id % kXcds;
    id = x * q + min(x, r) + id / kXcds;
  }
  const uint32_t n_rowtiles = (uint32_t)p.total_tiles;
  const int kvh = (int)fast_div(id, p.tiles_div);
  const int rowtile = (int)(id - (uint32_t)kvh * n_rowtiles);
  const int b = find_segment(meta.tile_start, meta.n, rowtile);
  const int q_tok0 = meta.start[b], lq = meta.len[b], k_tok0 = meta.kstart[b];
  const int jt = rowtile - meta.tile_start[b];
  const int dq = q_tok0 - k_tok0;  // the block's first token, counted in keys
  const int lk = dq + lq;          // keys up to the block's end

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 31, hf = lane >> 5;
  const int Gq = p.group;
  const int n_rows = lq * Gq;
  const int row0 = jt * kShortTileRows;
  const int last_row = min(n_rows, row0 + kShortTileRows) - 1;
  const int n_t = (dq + (int)fast_div((uint32_t)last_row, p.group_div)) / kBKeys + 1;
  const int wave_row0 = row0 + wave * 32;
  const int wave_last_row = min(n_rows, wave_row0 + 32) - 1;
  const int wave_n_t =
      wave_last_row >= wave_row0 ? (dq + (int)fast_div((uint32_t)wave_last_row, p.group_div)) / kBKeys + 1 : 0;
  const int first_key_wave = dq + (int)fast_div((uint32_t)wave_row0, p.group_div);
  const int my_row = min(wave_row0 + col, n_rows - 1);  // (lanes beyond the block's rows repeat its last row)
  const int my_tok = (int)fast_div((uint32_t)my_row, p.group_div);
  const int my_key = dq + my_tok;

  // ---- whole rows of q^ and dO for this wave, requested first (see the forward kernel) -----------
  auto walk_rows = [&](uint32_t st, uint32_t sh, auto &&visit) __attribute__((always_inline)) {
    const int wr_r0 = wave_row0 + lane / G::CPR;
    const int wr_tok0 = (int)fast_div((uint32_t)wr_r0, p.group_div);
    const int wr_g0 = wr_r0 - wr_tok0 * Gq;
    uint32_t off = (uint32_t)wr_tok0 * st + (uint32_t)wr_g0 * sh;
    int g = wr_g0;
    const uint32_t d_in = 4u * sh, d_wrap = st + (uint32_t)(4 - Gq) * sh;
#pragma unroll
    for (int u = 0; u < G::KCH; ++u) {
      visit(u, off, wr_r0);
#pragma unroll
      for (int s4 = 0; s4 < G::QRPI / 4; ++s4) {
        g += 4;
        const bool wrap = g >= Gq;
        g = wrap ? g - Gq : g;
        off += wrap ? d_wrap : d_in;
      }
    }
  };
  u32x4_t ld_q[G::KCH], ld_do[G::KCH];
  {
    const char *qbase = (const char *)(p.q + (int64_t)q_tok0 * p.q_st + (int64_t)(kvh * Gq) * p.q_sh);
    const uint32_t st = (uint32_t)p.q_st, sh = (uint32_t)p.q_sh;
    const uint32_t last_off = (uint32_t)(lq - 1) * st + (uint32_t)(Gq - 1) * sh;
    walk_rows(st, sh, [&](int u, uint32_t off, int wr_r0) __attribute__((always_inline)) {
      const uint32_t o = wr_r0 < n_rows - u * G::QRPI ? off : last_off;
      ld_q[u] = *reinterpret_cast<const u32x4_t *>(qbase + (o * 2u + (uint32_t)(lane % G::CPR) * 16u));
    });
  }
  {
    const char *dbase = (const char *)(bp.dout + (int64_t)q_tok0 * bp.do_st + (int64_t)(kvh * Gq) * bp.do_sh);
    const uint32_t st = (uint32_t)bp.do_st, sh = (uint32_t)bp.do_sh;
    const uint32_t last_off = (uint32_t)(lq - 1) * st + (uint32_t)(Gq - 1) * sh;
    walk_rows(st, sh, [&](int u, uint32_t off, int wr_r0) __attribute__((always_inline)) {
      const uint32_t o = wr_r0 < n_rows - u * G::QRPI ? off : last_off;
      ld_do[u] = *reinterpret_cast<const u32x4_t *>(dbase + (o * 2u + (uint32_t)(lane % G::CPR) * 16u));
    });
  }
  // ... and of O, for delta = rowsum(dO o O); this lane's row's log-sum-exp (to base-2 units below)
  u32x4_t ld_o[G::KCH];
  {
    const char *obase = (const char *)(bp.o + (int64_t)q_tok0 * bp.o_st + (int64_t)(kvh * Gq) * bp.o_sh);
    const uint32_t st = (uint32_t)bp.o_st, sh = (uint32_t)bp.o_sh;
    const uint32_t last_off = (uint32_t)(lq - 1) * st + (uint32_t)(Gq - 1) * sh;
    walk_rows(st, sh, [&](int u, uint32_t off, int wr_r0) __attribute__((always_inline)) {
      const uint32_t o = wr_r0 < n_rows - u * G::QRPI ? off : last_off;
      ld_o[u] = *reinterpret_cast<const u32x4_t *>(obase + (o * 2u + (uint32_t)(lane % G::CPR) * 16u));
    });
  }
  const float my_lse = bp.lse[(int64_t)(q_tok0 + my_tok) * p.n_q_heads + kvh * Gq + (my_row - my_tok * Gq)];
  __builtin_amdgcn_sched_barrier(0);

  // ---- per-lane LDS read offsets inside a tile ---------------------------------------------------
  uint32_t k_rd[G::KCH];  // rows as A operand: row `col`, chunk 2 kk + hf
#pragma unroll
  for (int kk = 0; kk < G::KCH; ++kk) k_rd[kk] = tile_ofs<D>(col, kk * 2 + hf);
  // transposed A operand (16-row step 0): 8-byte piece of row trow (+8), head dims 32 dt + ...
  uint32_t t_rd[2][G::DT];
  {
    const int trow = hf * 4 + ((lane & 15) >> 2);
#pragma unroll
    for (int dt = 0; dt < G::DT; ++dt) {
      const int byte = dt * 64 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
      t_rd[0][dt] = tile_ofs<D>(trow, byte >> 4) + (byte & 15);
      t_rd[1][dt] = tile_ofs<D>(trow + 8, byte >> 4) + (byte & 15);
    }
  }

  // ---- tile fill (K and V rows of 32 keys; rows beyond the valid ones repeat the last valid row) ----
  const char *k_base = (const char *)(p.kf + (int64_t)k_tok0 * p.kf_st + (int64_t)kvh * p.kf_sh);
  const char *v_base = (const char *)(p.vf + (int64_t)k_tok0 * p.vf_st + (int64_t)kvh * p.vf_sh);
  const uint32_t k_rb = (uint32_t)p.kf_st * 2u, v_rb = (uint32_t)p.vf_st * 2u;
  int c_row[G::IPW];
  uint32_t c_chunk[G::IPW];
#pragma unroll
  for (int u = 0; u < G::IPW; ++u) {
    const int row = (wave * G::IPW + u) * G::RPI + lane / G::CPR, pos = lane % G::CPR;
    c_row[u] = row;
    c_chunk[u] = (uint32_t)(pos ^ ((row / G::LPR) & (G::CPR - 1))) << 4;
  }
  const uint32_t lds_copy = (uint32_t)(uintptr_t)smem + wave * G::IPW * 1024;
  auto issue_copy = [&](int t, int buf) __attribute__((always_inline)) {
    const int valid = min(kBKeys, lk - t * kBKeys);
    const char *kp = k_base + (uint64_t)(uint32_t)(t * kBKeys) * (uint64_t)k_rb;
    const char *vp = v_base + (uint64_t)(uint32_t)(t * kBKeys) * (uint64_t)v_rb;
#pragma unroll
    for (int u = 0; u < G::IPW; ++u) {
      const uint32_t row = (uint32_t)min(c_row[u], valid - 1);
      lds_dma16(kp, row * k_rb + c_chunk[u], lds_copy + (uint32_t)buf * (2 * TB) + u * 1024);
      lds_dma16(vp, row * v_rb + c_chunk[u], lds_copy + (uint32_t)buf * (2 * TB) + TB + u * 1024);
    }
  };
  constexpr int kOpsPerTile = 2 * G::IPW;
  issue_copy(0, 0);  // (buffer 2 holds the waves' slices until the first barrier)
  if (1 < n_t) issue_copy(1, 1);
  __builtin_amdgcn_sched_barrier(0);
  dma_wait<0>();

  // ---- whole rows -> B-operand fragments (lane = row), 16 rows at a time through this wave's slice ----
  static_assert(kBWaves * 16 * G::ROWB <= 2 * TB, "the slices fit one tile buffer");
  const uint32_t s_ofs = 2 * (2 * TB) + wave * (16 * G::ROWB);
  auto rows_to_frags = [&](const u32x4_t (&ld)[G::KCH], bf16x8_t (&out)[G::KCH]) __attribute__((always_inline)) {
    u32x4_t got[2][G::KCH];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
      for (int u = 0; u < G::KCH / 2; ++u)
        *reinterpret_cast<__attribute__((address_space(3))) u32x4_t *>(
            smem + s_ofs + tile_ofs<D>(u * G::QRPI + lane / G::CPR, lane % G::CPR)) = ld[pass * (G::KCH / 2) + u];
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk)
        got[pass][kk] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t *>(
            smem + s_ofs + tile_ofs<D>(col & 15, kk * 2 + hf));
    }
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) {
      u32x4_t w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (col >> 4) ? got[1][kk][e] : got[0][kk][e];
      asm volatile("" : "+v"(w));
      out[kk] = __builtin_bit_cast(bf16x8_t, w);
    }
  };
  // delta of this wave's rows: a row's CPR lanes add up their pieces, one of them hands the sum over
  // through the slice to the lane that owns the row; the pair (L / ln 2, delta) also goes to memory in
  // packed-row order per KV head, where the dk/dv kernel finds the 32 pairs of a row tile side by side
  float2 my_ld;
  {
#pragma unroll
    for (int u = 0; u < G::KCH; ++u) {
      float part = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        part += bf16_lo(ld_o[u][e]) * bf16_lo(ld_do[u][e]) + bf16_hi(ld_o[u][e]) * bf16_hi(ld_do[u][e]);
#pragma unroll
      for (int m = 1; m < G::CPR; m <<= 1) part += __shfl_xor(part, m, 64);
      if (lane % G::CPR == 0)
        *reinterpret_cast<__attribute__((address_space(3))) float *>(smem + s_ofs + (u * G::QRPI + lane / G::CPR) * 4) = part;
    }
    const int r_in_wave = min(col, max(wave_last_row - wave_row0, 0));  // (lanes beyond the block's rows: its last row)
    my_ld.y = *reinterpret_cast<const __attribute__((address_space(3))) float *>(smem + s_ofs + r_in_wave * 4);
    my_ld.x = my_lse * kLog2e;
    if (hf == 0 && wave_row0 + col < n_rows) bp.ld[((int64_t)kvh * bp.T + q_tok0) * Gq + wave_row0 + col] = my_ld;
  }
  bf16x8_t qf[G::KCH], dof[G::KCH];
  rows_to_frags(ld_q, qf);
  rows_to_frags(ld_do, dof);

  f32x16_t acc[G::DT];
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[dt][v] = 0.f;

  // ---- the walk over the key tiles ---------------------------------------------------------------
  int buf = 0;
#pragma unroll 1
  for (int i = 0; i < n_t; ++i) {
    if (i + 1 < n_t) dma_wait<kOpsPerTile>(); else dma_wait<0>();
    wg_barrier();
    if (i + 2 < n_t) issue_copy(i + 2, buf == 0 ? 2 : buf - 1);
    if (i < wave_n_t) {
      const uint32_t kofs = (uint32_t)buf * (2 * TB), vofs = kofs + TB;
      // S'^T - L: the base-2 exponent of P;  dP^T - delta
      f32x16_t sacc, dpacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        sacc[v] = -my_ld.x;
        dpacc[v] = -my_ld.y;
      }
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk) {
        const bf16x8_t kfrag = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(smem + (k_rd[kk] + kofs));
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag, qf[kk], sacc, 0, 0, 0);
        const bf16x8_t vfrag = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(smem + (k_rd[kk] + vofs));
        dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfrag, dof[kk], dpacc, 0, 0, 0);
      }
      const int key0 = i * kBKeys;
      const int valid = min(kBKeys, lk - key0);
      if (key0 + kBKeys - 1 > first_key_wave || valid < kBKeys) {
        const int lim = min(my_key - key0 + 1, valid);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = (v >> 2) * 8 + hf * 4 + (v & 3);
          if (key >= lim) sacc[v] = -INFINITY;
        }
      }
      // dS^T = P^T o (dP^T - delta), rounded to bf16: the B operand of dq^^T += K^T dS^T
      bf16x8_t dsf[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        u32x4_t w;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float d0 = __builtin_amdgcn_exp2f(sacc[e * 8 + 2 * j]) * dpacc[e * 8 + 2 * j];
          const float d1 = __builtin_amdgcn_exp2f(sacc[e * 8 + 2 * j + 1]) * dpacc[e * 8 + 2 * j + 1];
          w[j] = pack_bf16(d0, d1);
        }
        dsf[e] = __builtin_bit_cast(bf16x8_t, w);
      }
#pragma unroll
      for (int kc = 0; kc < 2; ++kc)
#pragma unroll
        for (int dt = 0; dt < G::DT; ++dt) {
          typedef __attribute__((address_space(3))) s16x4_t lds_s16x4;
          typedef short s16x8_t __attribute__((ext_vector_type(8)));
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + (t_rd[0][dt] + kofs) + kc * 16 * G::ROWB));
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + (t_rd[1][dt] + kofs) + kc * 16 * G::ROWB));
          const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, both), dsf[kc], acc[dt], 0, 0, 0);
        }
    }
    buf = buf == kBBuf - 1 ? 0 : buf + 1;
  }

  // ---- epilogue: dq^ = scale * acc, turned back to dq with the row's entry of the pre-pass's table
  //      (which carries scale * log2 e: scale / (scale * log2 e) = ln 2 remains), bf16, as whole rows
  //      through each wave's slice of LDS -------------------------------------------------------------
  wg_barrier();
  int ln = lane;
  asm volatile("" : "+v"(ln));
  const int ecol = ln & 31, ehf = ln >> 5;
  rotate_back<D>(acc, reinterpret_cast<const f32x4_t *>(p.q_table + (int64_t)(q_tok0 + my_tok) * D), ehf,
                 p.rope_layout != 0, kLn2);
  lds_char *stage = smem + wave * (32 * G::ROWB);
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
      u32x2_t w;
      w[0] = pack_bf16(acc[dt][q4 * 4 + 0], acc[dt][q4 * 4 + 1]);
      w[1] = pack_bf16(acc[dt][q4 * 4 + 2], acc[dt][q4 * 4 + 3]);
      *reinterpret_cast<__attribute__((address_space(3))) u32x2_t *>(stage + tile_ofs<D>(ecol, dt * 4 + q4) + ehf * 8) = w;
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  {
    u32x4_t w[G::KCH];
#pragma unroll
    for (int u = 0; u < G::KCH; ++u)
      w[u] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t *>(
          stage + tile_ofs<D>(u * G::QRPI + ln / G::CPR, ln % G::CPR));
    char *obase = (char *)(bp.dq + (int64_t)q_tok0 * bp.dq_st + (int64_t)(kvh * Gq) * bp.dq_sh);
    walk_rows((uint32_t)bp.dq_st, (uint32_t)bp.dq_sh, [&](int u, uint32_t off, int wr_r0) __attribute__((always_inline)) {
      if (wr_r0 < n_rows - u * G::QRPI)
        *reinterpret_cast<u32x4_t *>(obase + (off * 2u + (uint32_t)(ln % G::CPR) * 16u)) = w[u];
    });
  }
}

// ---------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBThreads, 2) void bwd_dkv_kernel(AttnParams p, BwdKvMeta meta, BwdParams bp) {
  using G = BGeo<D>;
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char *smem = (lds_char *)smem_generic;
  // LDS map: buffer b = bytes [b BUFB, (b + 1) BUFB): a q^ tile, a dO tile (kKvRows packed query rows
  // each, i.e. RG groups of 32: two independent chains of products per iteration, which a single
  // wave per SIMD needs to keep the matrix pipe fed), then per wave 1 KB whose first kKvRows * 8
  // bytes hold the rows' (L / ln 2, delta)
  constexpr int RG = kKvRows / 32;
  constexpr uint32_t TB = RG * G::TILEB;
  constexpr uint32_t BUFB = 2 * TB + kBWaves * 1024;
  constexpr int IPW = RG * G::IPW;  // LDS-direct loads per wave, tile and tensor

  uint32_t id = blockIdx.x;
  {
    constexpr uint32_t kXcds = 8;
    const uint32_t n_wg = gridDim.x, q = n_wg / kXcds, r = n_wg % kXcds, x = id % kXcds;
    id = x * q + min(x, r) + id / kXcds;
  }
  const uint32_t n_keytiles = (uint32_t)p.total_tiles;
  const int kvh = (int)fast_div(id, p.tiles_div);
  const int keytile = (int)(id - (uint32_t)kvh * n_keytiles);
  const int b = find_segment(meta.tile_start, meta.n, keytile);
  const int k_tok0 = meta.start[b], lk = meta.len[b];  // the block that owns the keys
  const int f_tok0 = meta.fin_start[b], lf = meta.fin_len[b];  // its prompt's last block, if it is a passage
  const int k0 = (keytile - meta.tile_start[b]) * kShortTileRows;  // the workgroup's first key, inside the block

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 31, hf = lane >> 5;
  const int Gq = p.group;
  const int kw0 = k0 + wave * 32;  // this wave's first key
  const bool wave_has_keys = kw0 < lk;
  const int my_key = kw0 + col;    // (may lie beyond the block: such columns are never stored)

  // ---- query row tiles that see these keys: the block's own rows from the first key's token on,
  //      then every row of the prompt's last block ------------------------------------------------
  const int n_rows_a = lk * Gq, n_rows_f = lf * Gq;
  const int tile_a0 = (k0 * Gq) / kKvRows;
  const int n_a = (n_rows_a + kKvRows - 1) / kKvRows - tile_a0;
  const int n_t = n_a + (n_rows_f + kKvRows - 1) / kKvRows;

  // ---- this wave's keys as B operands: k^ and v rows, whole, then into fragments through LDS ----
  u32x4_t ld_k[G::KCH], ld_v[G::KCH];
  {
    const char *kb = (const char *)(p.kf + (int64_t)k_tok0 * p.kf_st + (int64_t)kvh * p.kf_sh);
    const char *vb = (const char *)(p.vf + (int64_t)k_tok0 * p.vf_st + (int64_t)kvh * p.vf_sh);
#pragma unroll
    for (int u = 0; u < G::KCH; ++u) {
      const uint32_t tok = (uint32_t)min(kw0 + u * G::QRPI + lane / G::CPR, lk - 1);
      ld_k[u] = *reinterpret_cast<const u32x4_t *>(kb + ((uint64_t)tok * (uint64_t)p.kf_st + (uint32_t)(lane % G::CPR) * 8u) * 2u);
      ld_v[u] = *reinterpret_cast<const u32x4_t *>(vb + ((uint64_t)tok * (uint64_t)p.vf_st + (uint32_t)(lane % G::CPR) * 8u) * 2u);
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // rows as A operand: row `col`, chunk 2 kk + hf, i.e. byte (32 kk) ^ row_x inside the row (worked
  // out at each use: eight more address registers would not fit two waves per SIMD)
  const uint32_t row_b = (uint32_t)col * G::ROWB;
  const uint32_t row_x = (uint32_t)(hf ^ ((col / G::LPR) & (G::CPR - 1))) << 4;
  uint32_t t_rd[2][G::DT];
  {
    const int trow = hf * 4 + ((lane & 15) >> 2);
#pragma unroll
    for (int dt = 0; dt < G::DT; ++dt) {
      const int byte = dt * 64 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
      t_rd[0][dt] = tile_ofs<D>(trow, byte >> 4) + (byte & 15);
      t_rd[1][dt] = tile_ofs<D>(trow + 8, byte >> 4) + (byte & 15);
    }
  }

  // ---- tile fill: kKvRows packed query rows of q^ and of dO, and the rows' (L, delta) ------------------
  const uint32_t q_st = (uint32_t)p.q_st, q_sh = (uint32_t)p.q_sh, do_st = (uint32_t)bp.do_st, do_sh = (uint32_t)bp.do_sh;
  const uint32_t lds_copy = (uint32_t)(uintptr_t)smem + wave * IPW * 1024;
  const uint32_t lds_ld = (uint32_t)(uintptr_t)smem + 2 * TB + wave * 1024;
  auto issue_copy = [&](int t, int buf) __attribute__((always_inline)) {
    const bool own = t < n_a;
    const int r0 = (own ? tile_a0 + t : t - n_a) * kKvRows;  // first packed row of the tile, inside its block
    const int tok0 = own ? k_tok0 : f_tok0;
    const int n_rows = own ? n_rows_a : n_rows_f;
    const char *qb = (const char *)(p.q + (int64_t)tok0 * p.q_st + (int64_t)(kvh * Gq) * p.q_sh);
    const char *db = (const char *)(bp.dout + (int64_t)tok0 * bp.do_st + (int64_t)(kvh * Gq) * bp.do_sh);
#pragma unroll
    for (int u = 0; u < IPW; ++u) {
      const int rt = (wave * IPW + u) * G::RPI + lane / G::CPR, pos = lane % G::CPR;
      const uint32_t r = (uint32_t)min(r0 + rt, n_rows - 1);  // rows beyond the block repeat its last row
      const uint32_t tok = fast_div(r, p.group_div), g = r - tok * (uint32_t)Gq;
      const uint32_t chunk = (uint32_t)(pos ^ ((rt / G::LPR) & (G::CPR - 1))) << 4;
      lds_dma16(qb, (tok * q_st + g * q_sh) * 2u + chunk, lds_copy + (uint32_t)buf * BUFB + u * 1024);
      lds_dma16(db, (tok * do_st + g * do_sh) * 2u + chunk, lds_copy + (uint32_t)buf * BUFB + TB + u * 1024);
    }
    // (L, delta) of the rows: contiguous in packed-row order, 16 bytes (two rows) per lane; every wave
    // fetches its own copy (the upper lanes re-read the same bytes), so that all waves count alike
    const char *lb = (const char *)(bp.ld + ((int64_t)kvh * bp.T + tok0) * Gq);
    const uint32_t r = (uint32_t)min(r0 + (lane & (kKvRows / 2 - 1)) * 2, n_rows - 2 + (n_rows & 1));
    lds_dma16(lb, (r & ~1u) * 8u, lds_ld + (uint32_t)buf * BUFB);
  };
  constexpr int kOpsPerTile = 2 * IPW + 1;
  if (0 < n_t) issue_copy(0, 0);
  if (1 < n_t) issue_copy(1, 1);
  __builtin_amdgcn_sched_barrier(0);
  dma_wait<0>();

  // ---- k^ and v rows -> B-operand fragments through this wave's slice of buffer 2 -------------------
  static_assert(kBWaves * 16 * G::ROWB <= 2 * TB, "the slices fit the tiles of one buffer");
  static_assert(kKvRows * 8 <= 1024 && kKvRows / 2 <= 64, "a wave's (L, delta) copy fits its 1 KB");
  const uint32_t s_ofs = 2 * BUFB + wave * (16 * G::ROWB);
  auto rows_to_frags = [&](const u32x4_t (&ld)[G::KCH], bf16x8_t (&out)[G::KCH]) __attribute__((always_inline)) {
    u32x4_t got[2][G::KCH];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
      for (int u = 0; u < G::KCH / 2; ++u)
        *reinterpret_cast<__attribute__((address_space(3))) u32x4_t *>(
            smem + s_ofs + tile_ofs<D>(u * G::QRPI + lane / G::CPR, lane % G::CPR)) = ld[pass * (G::KCH / 2) + u];
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk)
        got[pass][kk] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t *>(
            smem + s_ofs + tile_ofs<D>(col & 15, kk * 2 + hf));
    }
#pragma unroll
    for (int kk = 0; kk < G::KCH; ++kk) {
      u32x4_t w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (col >> 4) ? got[1][kk][e] : got[0][kk][e];
      asm volatile("" : "+v"(w));
      out[kk] = __builtin_bit_cast(bf16x8_t, w);
    }
  };
  bf16x8_t kf[G::KCH], vf[G::KCH];
  rows_to_frags(ld_k, kf);
  rows_to_frags(ld_v, vf);

  f32x16_t dk[G::DT], dv[G::DT];
#pragma unroll
  for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      dk[dt][v] = 0.f;
      dv[dt][v] = 0.f;
    }

  // ---- the walk over the query row tiles ------------------------------------------------------------
  int buf = 0;
#pragma unroll 1
  for (int i = 0; i < n_t; ++i) {
    if (i + 1 < n_t) dma_wait<kOpsPerTile>(); else dma_wait<0>();
    wg_barrier();
    if (i + 2 < n_t) issue_copy(i + 2, buf == 0 ? 2 : buf - 1);
    const bool own = i < n_a;
    const int r0 = (own ? tile_a0 + i : i - n_a) * kKvRows;
    const int n_rows = own ? n_rows_a : n_rows_f;
    // a tile of the block's own rows whose tokens all lie before this wave's first key sees none of them
    const int last_tok = (int)fast_div((uint32_t)min(r0 + kKvRows - 1, n_rows - 1), p.group_div);
    if (wave_has_keys && !(own && last_tok < kw0)) {
      const uint32_t qofs = (uint32_t)buf * BUFB, dofs = qofs + TB;
      uint32_t rx = row_x;
      asm volatile("" : "+v"(rx));  // (keeps the eight offsets below from being carried through the loop)
      // The accumulators start at minus the rows' log-sum-exp and minus their delta, so that the
      // products come out as the exponent of P and as dP - delta.  Register v of an accumulator is
      // row (v >> 2) * 8 + hf * 4 + (v & 3) of the group: four runs of four rows, two pairs per 16 bytes.
      f32x16_t sacc[RG], dpacc[RG];
#pragma unroll
      for (int rg = 0; rg < RG; ++rg)
#pragma unroll
        for (int run = 0; run < 4; ++run)
#pragma unroll
          for (int h2 = 0; h2 < 2; ++h2) {
            const f32x4_t two = *reinterpret_cast<const __attribute__((address_space(3))) f32x4_t *>(
                smem + 2 * TB + wave * 1024 + qofs + (rg * 32 + run * 8 + hf * 4 + h2 * 2) * 8);
            sacc[rg][run * 4 + h2 * 2] = -two[0];
            dpacc[rg][run * 4 + h2 * 2] = -two[1];
            sacc[rg][run * 4 + h2 * 2 + 1] = -two[2];
            dpacc[rg][run * 4 + h2 * 2 + 1] = -two[3];
          }
#pragma unroll
      for (int kk = 0; kk < G::KCH; ++kk)
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
          const bf16x8_t qfrag = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(
              smem + (row_b + (((uint32_t)kk * 32u) ^ rx) + qofs) + rg * 32 * G::ROWB);
          sacc[rg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfrag, kf[kk], sacc[rg], 0, 0, 0);
          const bf16x8_t dfrag = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t *>(
              smem + (row_b + (((uint32_t)kk * 32u) ^ rx) + dofs) + rg * 32 * G::ROWB);
          dpacc[rg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dfrag, vf[kk], dpacc[rg], 0, 0, 0);
        }
      // which rows this key may not see: rows beyond the block, and (own block) tokens before the key
      const bool ragged = r0 + kKvRows > n_rows;
      const int first_tok = (int)fast_div((uint32_t)r0, p.group_div);
      const bool diagonal = own && first_tok < kw0 + 32;
      bf16x8_t pf[2 * RG], dsf[2 * RG];
#pragma unroll
      for (int rg = 0; rg < RG; ++rg) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          u32x4_t wp, wd;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            float pv[2], dsv[2];
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
              const int v = e * 8 + 2 * j + h2;
              float pr = __builtin_amdgcn_exp2f(sacc[rg][v]);
              const int row = r0 + rg * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
              if (ragged && row >= n_rows) pr = 0.f;
              if (diagonal && (int)fast_div((uint32_t)row, p.group_div) < my_key) pr = 0.f;
              pv[h2] = pr;
              dsv[h2] = pr * dpacc[rg][v];
            }
            wp[j] = pack_bf16(pv[0], pv[1]);
            wd[j] = pack_bf16(dsv[0], dsv[1]);
          }
          pf[rg * 2 + e] = __builtin_bit_cast(bf16x8_t, wp);
          dsf[rg * 2 + e] = __builtin_bit_cast(bf16x8_t, wd);
        }
      }
#pragma unroll
      for (int kc = 0; kc < 2 * RG; ++kc)
#pragma unroll
        for (int dt = 0; dt < G::DT; ++dt) {
          typedef __attribute__((address_space(3))) s16x4_t lds_s16x4;
          typedef short s16x8_t __attribute__((ext_vector_type(8)));
          const s16x4_t dlo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + (t_rd[0][dt] + dofs) + kc * 16 * G::ROWB));
          const s16x4_t dhi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + (t_rd[1][dt] + dofs) + kc * 16 * G::ROWB));
          const s16x8_t dboth = __builtin_shufflevector(dlo, dhi, 0, 1, 2, 3, 4, 5, 6, 7);
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, dboth), pf[kc], dv[dt], 0, 0, 0);
          const s16x4_t qlo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + (t_rd[0][dt] + qofs) + kc * 16 * G::ROWB));
          const s16x4_t qhi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + (t_rd[1][dt] + qofs) + kc * 16 * G::ROWB));
          const s16x8_t qboth = __builtin_shufflevector(qlo, qhi, 0, 1, 2, 3, 4, 5, 6, 7);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, qboth), dsf[kc], dk[dt], 0, 0, 0);
        }
    }
    buf = buf == kBBuf - 1 ? 0 : buf + 1;
  }

  // ---- epilogue: dV as it is; dk^ = ln 2 * acc (the q^ tiles carry scale * log2 e), turned back to dk
  //      with the key's entry of the pre-pass's table (which carries scale * log2 e once more); bf16,
  //      whole rows ------------------------------------------------------------------------------------
  wg_barrier();
  int ln = lane;
  asm volatile("" : "+v"(ln));
  const int ecol = ln & 31, ehf = ln >> 5;
  rotate_back<D>(dk, reinterpret_cast<const f32x4_t *>(p.q_table + (int64_t)(k_tok0 + min(kw0 + ecol, lk - 1)) * D), ehf,
                 p.rope_layout != 0, kLn2 / p.scale_log2e);
  lds_char *stage = smem + wave * (32 * G::ROWB);
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
    for (int dt = 0; dt < G::DT; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        const f32x16_t &a = pass == 0 ? dv[dt] : dk[dt];
        u32x2_t w;
        w[0] = pack_bf16(a[q4 * 4 + 0], a[q4 * 4 + 1]);
        w[1] = pack_bf16(a[q4 * 4 + 2], a[q4 * 4 + 3]);
        *reinterpret_cast<__attribute__((address_space(3))) u32x2_t *>(stage + tile_ofs<D>(ecol, dt * 4 + q4) + ehf * 8) = w;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint16_t *dst = pass == 0 ? bp.dv : bp.dk;
    const int64_t st = pass == 0 ? bp.dv_st : bp.dk_st, sh = pass == 0 ? bp.dv_sh : bp.dk_sh;
#pragma unroll
    for (int u = 0; u < G::KCH; ++u) {
      const int rr = u * G::QRPI + ln / G::CPR;
      const u32x4_t w = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t *>(stage + tile_ofs<D>(rr, ln % G::CPR));
      if (kw0 + rr < lk)
        *reinterpret_cast<u32x4_t *>(dst + (int64_t)(k_tok0 + kw0 + rr) * st + (int64_t)kvh * sh + (ln % G::CPR) * 8) = w;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

template <int D>
hipError_t launch_dkv_t(const AttnParams &p, const BwdKvMeta &meta, const BwdParams &bp, hipStream_t stream) {
  const int64_t n_wg = (int64_t)p.total_tiles * p.n_kv_heads;
  if (n_wg == 0) return hipSuccess;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  constexpr size_t lds = (size_t)kBBuf * (2 * (kKvRows / 32) * BGeo<D>::TILEB + kBWaves * 1024);
  static_assert(lds <= 160 * 1024, "gfx950 has 160 KB of LDS per workgroup");
  // more than 64 KB of dynamic LDS has to be asked for once per kernel (setting it twice, from two
  // host threads at once, is harmless)
  static std::atomic<bool> raised{false};
  if (lds > 64 * 1024 && !raised.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&bwd_dkv_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    raised.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((bwd_dkv_kernel<D>), dim3((unsigned)n_wg), dim3(kBThreads), lds, stream, p, meta, bp);
  return hipGetLastError();
}

template <int D>
hipError_t launch_dq_t(const AttnParams &p, const PromptMeta &meta, const BwdParams &bp, hipStream_t stream) {
  const int64_t n_wg = (int64_t)p.total_tiles * p.n_kv_heads;
  if (n_wg == 0) return hipSuccess;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  constexpr size_t lds = (size_t)2 * kBBuf * BGeo<D>::TILEB;
  static_assert(lds <= 64 * 1024, "fits the default dynamic LDS limit");
  hipLaunchKernelGGL((bwd_dq_kernel<D>), dim3((unsigned)n_wg), dim3(kBThreads), lds, stream, p, meta, bp);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_dkv(const AttnParams &p, const BwdKvMeta &meta, const BwdParams &bp, hipStream_t stream) {
  if (p.head_dim == 128) return launch_dkv_t<128>(p, meta, bp, stream);
  if (p.head_dim == 64) return launch_dkv_t<64>(p, meta, bp, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_bwd_dq(const AttnParams &p, const PromptMeta &meta, const BwdParams &bp, hipStream_t stream) {
  if (p.head_dim == 128) return launch_dq_t<128>(p, meta, bp, stream);
  if (p.head_dim == 64) return launch_dq_t<64>(p, meta, bp, stream);
  return hipErrorInvalidValue;
}

}  // namespace ba
