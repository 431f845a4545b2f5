// C boundary, the final block straight from a table of cached blocks (Section 2.3 Eq. 2-3 folded into
// Section 2.5): the block-table launches, and the gathered route for short blocks.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <type_traits>
#include <vector>

#include "ba_api_common.h"

namespace {
using ba::align256;
using ba::check_heads;
using ba::check_offsets;
using ba::check_prompt_blocks;
using ba::fail;
using ba::FinalPlan;
using ba::BlocksPlan;
using ba::device_fail;
using ba::num_cus;
using namespace ba::api;
}  // namespace
// ------------------------------------------------------------------------------------------
namespace {

struct BlocksCall {
  const ba_heads *heads;
  const ba::RopeTable *rt;
  const ba_tensor *q_f;
  uint16_t *q_ws;
  const ba_tensor *k_f;
  const ba_tensor *kf_use;
  float *rot_ws;
  int32_t n_prompts;
  const int32_t *cu_q, *cu_blk, *blk_tok_off, *blk_len, *blk_old_pos0, *blk_new_pos0, *q_pos0;
  hipStream_t stream;
  int max_nt;  // longest walk of the call, key tiles
};

// Launches of at most MetaT::kPrompts prompts and MetaT::kBlocks non-empty blocks each: the RoPE
// pre-pass (fresh q and k of the chunk, rotations of its blocks), then the attention core.
template <typename MetaT, typename RotsT>
int32_t run_final_blocks(const BlocksCall &c, ba::AttnParams ap) {
  const int D = c.heads->head_dim, G = c.heads->n_q_heads / c.heads->n_kv_heads;
  std::vector<MetaT> metas(1);
  std::vector<RotsT> rots(1);
  int n0 = 0;
  int64_t rot_base = 0, tile_base = 0;
  while (n0 < c.n_prompts) {
    MetaT &meta = metas[0];
    RotsT &rr = rots[0];
    memset(&meta, 0, sizeof(meta));
    memset(&rr, 0, sizeof(rr));
    int np = 0, nb = 0;
    int64_t tiles = 0;
    std::vector<int32_t> pos0;
    while (n0 + np < c.n_prompts && np < MetaT::kPrompts) {
      const int n = n0 + np;
      int cnt = 0;
      for (int b = c.cu_blk[n]; b < c.cu_blk[n + 1]; ++b) cnt += c.blk_len[b] > 0;
      if (nb + cnt > MetaT::kBlocks) break;  // (a single prompt always fits: checked by the plan)
      meta.cu_q[np] = c.cu_q[n];
      meta.cu_blk[np] = nb;
      meta.tile_start[np] = (int32_t)tiles;
      int32_t ctx_tiles = 0;
      int64_t run = 0;  // the prompt's context so far = default position of the next block
      for (int b = c.cu_blk[n]; b < c.cu_blk[n + 1]; ++b) {
        const int32_t new0 = c.blk_new_pos0 ? c.blk_new_pos0[b] : (int32_t)run;
        run += c.blk_len[b];
        if (c.blk_len[b] == 0) continue;
        meta.blk_off[nb] = c.blk_tok_off[b];
        meta.blk_len[nb] = c.blk_len[b];
        meta.blk_tile0[nb] = ctx_tiles;
        ctx_tiles += (c.blk_len[b] + ba::kTileKeys - 1) / ba::kTileKeys;
        // the queries are turned back by the block's shift: angle = -(new - old) positions
        rr.angle[nb] = -(new0 - (c.blk_old_pos0 ? c.blk_old_pos0[b] : 0));
        ++nb;
      }
      meta.ctx_tiles[np] = ctx_tiles;
      pos0.push_back(c.q_pos0 ? c.q_pos0[n] : (int32_t)run);
      tiles += ((int64_t)(c.cu_q[n + 1] - c.cu_q[n]) * G + ba::kTileRows - 1) / ba::kTileRows;
      ++np;
    }
    meta.n = np;
    meta.cu_q[np] = c.cu_q[n0 + np];
    meta.cu_blk[np] = nb;
    meta.tile_start[np] = (int32_t)tiles;
    meta.rot_base = (int32_t)rot_base;
    ap.total_tiles = (int32_t)tiles;
    ap.tile_base = (int32_t)tile_base;
    tile_base += tiles;
    {
      int32_t rc_cuts = ba::plan_split_cuts(c.heads->xcd_speed, tiles, c.heads->n_kv_heads, ap.n_splits, c.max_nt, num_cus(),
                                            ba::final_q_bytes_per_kv_head(c.heads, c.cu_q[c.n_prompts]), ap.split_cut,
                                            &ap.use_cuts, &ap.kv_group, &ap.xcd_runs);
      if (rc_cuts) return rc_cuts;
    }
    const ba::RopeRots *big = nullptr;
    const ba::RopeRotsSmall *small = nullptr;
    if constexpr (std::is_same<RotsT, ba::RopeRots>::value) big = &rr; else small = &rr;
    int32_t rc = run_rope_prepass(c.heads, *c.rt, c.q_f, c.q_ws, c.k_f, c.kf_use, np, meta.cu_q, pos0.data(), c.stream,
                                  big, small, c.rot_ws + rot_base * D, nb);
    if (rc) return rc;
    hipError_t e;
    {
      ProfileScope ps(BA_PROFILE_ATTENTION, c.stream);
      e = ba::launch_attn_final_blocks(ap, meta, c.stream);
    }
    if (e != hipSuccess) return device_fail(e, "final-block (cached) attention launch");
    rot_base += nb;
    n0 += np;
  }
  return BA_OK;
}

}  // namespace

extern "C" {

size_t ba_final_block_attention_cached_workspace_bytes(const ba_heads *heads, int32_t n_prompts,
                                                       const int32_t *cu_q, const int32_t *cu_blk,
                                                       const int32_t *blk_len, int32_t have_k_f_rot_out,
                                                       int32_t gather_below) {
  if (check_heads(heads, true) != BA_OK) return 0;
  BlocksPlan pl;
  if (ba::plan_final_blocks(heads, n_prompts, cu_q, cu_blk, blk_len, have_k_f_rot_out != 0, gather_below, num_cus(), &pl) != BA_OK)
    return 0;
  return pl.total();
}

int32_t ba_final_block_attention_cached(const ba_heads *heads, const ba_tensor *q_f, const ba_tensor *k_cache,
                                        const ba_tensor *v_cache, const ba_tensor *k_f, const ba_tensor *v_f,
                                        const ba_tensor *o_out, const ba_tensor *k_f_rot_out, int32_t n_prompts,
                                        const int32_t *cu_q, const int32_t *cu_blk, const int32_t *blk_tok_off,
                                        const int32_t *blk_len, const int32_t *blk_old_pos0,
                                        const int32_t *blk_new_pos0, const int32_t *q_pos0,
                                        int32_t gather_below, void *ws, size_t ws_bytes, void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  int32_t rc;
  if ((rc = check_heads(heads, true))) return rc;
  const int D = heads->head_dim;
  BlocksPlan pl;
  if ((rc = ba::plan_final_blocks(heads, n_prompts, cu_q, cu_blk, blk_len, k_f_rot_out != nullptr, gather_below, num_cus(), &pl)))
    return rc;
  if (n_prompts == 0) return BA_OK;
  if ((rc = check_tensor(q_f, "q_f", false, D, heads->n_q_heads))) return rc;
  if ((rc = check_tensor(k_f, "k_f", false, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(v_f, "v_f", false, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(o_out, "o_out", false, D, heads->n_q_heads))) return rc;
  if (pl.n_blocks > 0) {
    if (!blk_tok_off) return fail(BA_ERR_INVALID_ARG, "blk_tok_off is null");
    for (int b = 0; b < cu_blk[n_prompts]; ++b)
      if (blk_len[b] > 0 && blk_tok_off[b] < 0) return fail(BA_ERR_INVALID_ARG, "block %d: negative cache offset", b);
    if ((rc = check_tensor(k_cache, "k_cache", false, D, heads->n_kv_heads))) return rc;
    if ((rc = check_tensor(v_cache, "v_cache", false, D, heads->n_kv_heads))) return rc;
  }
  if (k_f_rot_out && (rc = check_tensor(k_f_rot_out, "k_f_rot_out", false, D, heads->n_kv_heads))) return rc;
  if (!ws || ws_bytes < pl.total() || ((uintptr_t)ws & 255))
    return fail(BA_ERR_WORKSPACE, "final block (cached): 256-byte aligned workspace of %zu bytes needed, %zu given",
                pl.total(), ws_bytes);

  if (pl.gather) {
    // non-empty blocks in prompt order: where they lie in the cache, where they go, and their positions
    std::vector<int32_t> src, dst, len, oldp, newp, zero;
    for (int n = 0; n < n_prompts; ++n) {
      int32_t at = pl.cu_ctx[n], pos = 0;
      for (int b = cu_blk[n]; b < cu_blk[n + 1]; ++b) {
        if (blk_len[b] == 0) continue;
        src.push_back(blk_tok_off[b]);
        dst.push_back(at);
        len.push_back(blk_len[b]);
        oldp.push_back(blk_old_pos0 ? blk_old_pos0[b] : 0);
        newp.push_back(blk_new_pos0 ? blk_new_pos0[b] : pos);
        at += blk_len[b];
        pos += blk_len[b];
      }
    }
    zero.assign(src.size(), 0);
    ba_tensor kg, vg;
    kg.ptr = ws;
    kg.stride_head = D;
    kg.stride_tok = (int64_t)heads->n_kv_heads * D;
    kg.dtype = BA_DTYPE_BF16;
    vg = kg;
    vg.ptr = (char *)ws + align256(pl.gather_kv_bytes);
    const int nb = (int)src.size();
    const int64_t v_after_k = ((const char *)v_cache->ptr - (const char *)k_cache->ptr) / 2;  // in elements
    if (k_cache->stride_tok == v_cache->stride_tok && k_cache->stride_head == v_cache->stride_head) {
      // One launch for both: the values ride along as a second "layer" of the key cache (the layer
      // strides are the distances between the two tensors) that is copied, not rotated.
      ba::RopeTable rt;
      build_rope_table(heads, &rt);
      ba::ReencParams rp;
      memset(&rp, 0, sizeof(rp));
      rp.src = k_cache->ptr;
      rp.dst = kg.ptr;
      rp.src_st = k_cache->stride_tok;
      rp.src_sh = k_cache->stride_head;
      rp.dst_st = kg.stride_tok;
      rp.dst_sh = kg.stride_head;
      rp.src_sl = v_after_k;
      rp.dst_sl = (int64_t)(align256(pl.gather_kv_bytes) / 2);
      rp.n_layers = 2;
      rp.n_kv_heads = heads->n_kv_heads;
      rp.head_dim = D;
      rp.dtype = BA_DTYPE_BF16;
      rp.layout = heads->rope_layout;
      rp.mode = BA_REENC_SHIFT;
      rp.copy_from_layer = 1;
      if ((rc = run_reencode(rp, rt, nb, src.data(), dst.data(), len.data(), oldp.data(), newp.data(), stream)))
        return rc;
    } else {
      if ((rc = ba_reencode_positions(heads, k_cache, &kg, 1, 0, 0, nb, src.data(), dst.data(), len.data(), oldp.data(),
                                      newp.data(), BA_REENC_SHIFT, stream_)))
        return rc;
      // (a shift of zero positions is a plain copy)
      if ((rc = ba_reencode_positions(heads, v_cache, &vg, 1, 0, 0, nb, src.data(), dst.data(), len.data(), zero.data(),
                                      zero.data(), BA_REENC_SHIFT, stream_)))
        return rc;
    }
    return ba_final_block_attention(heads, q_f, &kg, &vg, k_f, v_f, o_out, k_f_rot_out, n_prompts, cu_q,
                                    pl.cu_ctx.data(), q_pos0, BA_ROPE_APPLY,
                                    (char *)ws + 2 * align256(pl.gather_kv_bytes), pl.gather_final_bytes, stream_);
  }

  char *wsp = (char *)ws;
  void *kf_ws = wsp;
  wsp += align256(pl.kf_bytes);
  uint16_t *q_ws = (uint16_t *)wsp;
  wsp += align256(pl.q_bytes);
  float *rot_ws = (float *)wsp;
  wsp += align256(pl.rot_bytes);
  uint16_t *part_o = (uint16_t *)wsp;
  wsp += align256(pl.part_o_bytes);
  float *part_ml = (float *)wsp;
  wsp += align256(pl.part_ml_bytes);
  int32_t *part_idx = (int32_t *)wsp;

  ba::RopeTable rt;
  build_rope_table(heads, &rt);

  ba_tensor kf_use = *k_f;
  if (k_f_rot_out) {
    kf_use = *k_f_rot_out;
  } else {
    kf_use.ptr = kf_ws;
    kf_use.stride_head = D;
    kf_use.stride_tok = (int64_t)heads->n_kv_heads * D;
  }

  const int G = heads->n_q_heads / heads->n_kv_heads;
  ba::AttnParams ap;
  memset(&ap, 0, sizeof(ap));
  ap.q = q_ws;
  ap.q_st = (int64_t)heads->n_q_heads * D;
  ap.q_sh = D;
  ap.kf = (const uint16_t *)kf_use.ptr;
  ap.kf_st = kf_use.stride_tok;
  ap.kf_sh = kf_use.stride_head;
  ap.vf = (const uint16_t *)v_f->ptr;
  ap.vf_st = v_f->stride_tok;
  ap.vf_sh = v_f->stride_head;
  if (pl.n_blocks > 0) {
    ap.kc = (const uint16_t *)k_cache->ptr;
    ap.kc_st = k_cache->stride_tok;
    ap.kc_sh = k_cache->stride_head;
    ap.vc = (const uint16_t *)v_cache->ptr;
    ap.vc_st = v_cache->stride_tok;
    ap.vc_sh = v_cache->stride_head;
  } else {
    ap.kc = ap.kf;
    ap.kc_st = ap.kf_st;
    ap.kc_sh = ap.kf_sh;
    ap.vc = ap.vf;
    ap.vc_st = ap.vf_st;
    ap.vc_sh = ap.vf_sh;
  }
  ap.o = (uint16_t *)o_out->ptr;
  ap.o_st = o_out->stride_tok;
  ap.o_sh = o_out->stride_head;
  ap.part_o = part_o;
  ap.part_ml = part_ml;
  ap.part_idx = part_idx;
  ap.part_units = pl.total_tiles * heads->n_kv_heads * (ba::kTileRows / 32);
  ap.n_q_heads = heads->n_q_heads;
  ap.n_kv_heads = heads->n_kv_heads;
  ap.group = G;
  ap.group_div = ba::make_fast_div((uint32_t)G);
  ap.head_dim = D;
  ap.scale_log2e = scale_log2e(heads);
  ap.q_ready = 1;
  ap.rope_layout = heads->rope_layout;
  ap.blk_rot = rot_ws;
  ap.n_splits = pl.n_splits;

  BlocksCall call{heads, &rt, q_f, q_ws, k_f, &kf_use, rot_ws, n_prompts, cu_q, cu_blk, blk_tok_off, blk_len,
                  blk_old_pos0, blk_new_pos0, q_pos0, stream, pl.max_nt};
  if (n_prompts <= ba::kBlkSmallPrompts && pl.n_blocks <= ba::kBlkSmallBlocks)
    rc = run_final_blocks<ba::FinalBlocksMetaSmall, ba::RopeRotsSmall>(call, ap);
  else
    rc = run_final_blocks<ba::FinalBlocksMeta, ba::RopeRots>(call, ap);
  if (rc) return rc;
  if (pl.n_splits > 1) {
    hipError_t e;
    {
      ProfileScope ps(BA_PROFILE_COMBINE, stream);
      e = ba::launch_combine(ap, stream);
    }
    if (e != hipSuccess) return device_fail(e, "split combine launch");
  }
  return BA_OK;
}

}  // extern "C"

