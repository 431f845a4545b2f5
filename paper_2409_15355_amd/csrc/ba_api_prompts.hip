// C boundary, whole prompts under the Block-attention mask (Section 2.4): forward and backward entry
// points, and the route through zero-padded phantom heads for groups of fewer than four query heads.
#include <math.h>
#include <string.h>

#include <algorithm>
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

// ---- fewer than four query heads per KV head in the whole-prompt calls: run as groups of four --------
constexpr int kPadGroup = 4;

// A packed [T][n_kv_heads * 4][D] bf16 tensor in the workspace.
ba_tensor padded_tensor(void *ptr, const ba_heads *h) {
  ba_tensor t;
  t.ptr = ptr;
  t.stride_head = h->head_dim;
  t.stride_tok = (int64_t)h->n_kv_heads * kPadGroup * h->head_dim;
  t.dtype = BA_DTYPE_BF16;
  return t;
}
size_t padded_rows_bytes(const ba_heads *h, size_t T) { return align256(T * h->n_kv_heads * kPadGroup * h->head_dim * 2); }
size_t padded_lse_bytes(const ba_heads *h, size_t T) { return align256(T * h->n_kv_heads * kPadGroup * 4); }
ba_heads padded_heads(const ba_heads *h) {
  ba_heads p = *h;
  p.n_q_heads = h->n_kv_heads * kPadGroup;
  p.q_to_kv = nullptr;  // (the caller's map, if any, has been checked to be the default one)
  return p;
}
int32_t move_heads(const ba_heads *h, const ba_tensor *real, void *padded, int64_t T, bool to_padded, hipStream_t stream,
                   const char *what) {
  ba::HeadPadParams pp;
  memset(&pp, 0, sizeof(pp));
  pp.real = real->ptr;
  pp.real_st = real->stride_tok;
  pp.real_sh = real->stride_head;
  pp.padded = padded;
  pp.padded_sh = h->head_dim;
  pp.padded_st = (int64_t)h->n_kv_heads * kPadGroup * h->head_dim;
  pp.tokens = T;
  pp.n_kv_heads = h->n_kv_heads;
  pp.group = h->n_q_heads / h->n_kv_heads;
  pp.group_padded = kPadGroup;
  pp.chunks = h->head_dim * 2 / 16;
  pp.elt = 2;
  hipError_t e = ba::launch_pad_heads(pp, to_padded, stream);
  if (e != hipSuccess) return device_fail(e, what);
  return BA_OK;
}

}  // namespace

extern "C" {
// ------------------------------------------------------------------------------------------
size_t ba_block_attention_prompts_workspace_bytes(const ba_heads *heads, int32_t n_prompts, const int32_t *cu_blk,
                                                  const int32_t *block_offsets, int32_t rope_mode,
                                                  int32_t have_k_rot_out) {
  if (check_heads(heads, true) != BA_OK || check_prompt_blocks(n_prompts, cu_blk, block_offsets) != BA_OK) return 0;
  const size_t T = (size_t)block_offsets[cu_blk[n_prompts]];
  size_t pad_bytes = 0;
  if (heads->n_q_heads / heads->n_kv_heads < kPadGroup)  // padded q and o, padded log-sum-exps (see head_pad.hip)
    pad_bytes = 2 * padded_rows_bytes(heads, T) + padded_lse_bytes(heads, T);
  if (rope_mode != BA_ROPE_APPLY) return pad_bytes;
  const size_t k_bytes = have_k_rot_out ? 0 : align256(T * heads->n_kv_heads * heads->head_dim * 2);
  return pad_bytes + k_bytes + align256(T * heads->head_dim * 4);  // rotated K; scale * (cos, sin) per token and pair
}

int32_t ba_block_attention_prompts(const ba_heads *heads, const ba_tensor *q, const ba_tensor *k, const ba_tensor *v,
                                   const ba_tensor *o_out, const ba_tensor *k_rot_out, float *lse_out,
                                   int32_t n_prompts, const int32_t *cu_blk, const int32_t *block_offsets,
                                   int32_t rope_mode, void *ws, size_t ws_bytes, void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  int32_t rc;
  if ((rc = check_heads(heads, true))) return rc;
  if ((rc = check_prompt_blocks(n_prompts, cu_blk, block_offsets))) return rc;
  const int n_blocks = cu_blk[n_prompts];
  const int D = heads->head_dim;
  if ((rc = check_tensor(q, "q", false, D, heads->n_q_heads))) return rc;
  if ((rc = check_tensor(k, "k", false, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(v, "v", false, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(o_out, "o_out", false, D, heads->n_q_heads))) return rc;
  if (rope_mode != BA_ROPE_NONE && rope_mode != BA_ROPE_APPLY)
    return fail(BA_ERR_INVALID_ARG, "rope_mode %d unknown", rope_mode);
  if (k_rot_out) {
    if (rope_mode != BA_ROPE_APPLY) return fail(BA_ERR_INVALID_ARG, "k_rot_out needs rope_mode BA_ROPE_APPLY");
    if ((rc = check_tensor(k_rot_out, "k_rot_out", false, D, heads->n_kv_heads))) return rc;
  }
  if (lse_out && ((uintptr_t)lse_out & 3)) return fail(BA_ERR_ALIGNMENT, "lse_out must be 4-byte aligned");
  const int64_t T = block_offsets[n_blocks];
  const int G = heads->n_q_heads / heads->n_kv_heads;
  if (T == 0) return BA_OK;
  // what the kernel of this call is built for (see its header): groups of at least four query heads
  // per KV head, and blocks whose row offsets fit 32 bits
  int64_t max_len = 0;
  for (int b = 0; b < n_blocks; ++b) max_len = std::max<int64_t>(max_len, (int64_t)block_offsets[b + 1] - block_offsets[b]);
  const int64_t widest = std::max(std::max(q->stride_tok, o_out->stride_tok),
                                  (int64_t)G * std::max(q->stride_head, o_out->stride_head));
  if (G < kPadGroup) {
    // run as groups of four: padded q in, padded o and log-sum-exps out, through the workspace
    const size_t need =
        ba_block_attention_prompts_workspace_bytes(heads, n_prompts, cu_blk, block_offsets, rope_mode, k_rot_out != nullptr);
    if (!ws || ws_bytes < need || ((uintptr_t)ws & 255))
      return fail(BA_ERR_WORKSPACE, "whole prompts: 256-byte aligned workspace of %zu bytes needed, %zu given", need,
                  ws_bytes);
    const ba_heads h4 = padded_heads(heads);
    char *wsp = (char *)ws;
    const ba_tensor q4 = padded_tensor(wsp, heads);
    wsp += padded_rows_bytes(heads, (size_t)T);
    const ba_tensor o4 = padded_tensor(wsp, heads);
    wsp += padded_rows_bytes(heads, (size_t)T);
    float *lse4 = (float *)wsp;
    wsp += padded_lse_bytes(heads, (size_t)T);
    if ((rc = move_heads(heads, q, q4.ptr, T, true, stream, "whole prompts: head padding launch"))) return rc;
    if ((rc = ba_block_attention_prompts(&h4, &q4, k, v, &o4, k_rot_out, lse_out ? lse4 : nullptr, n_prompts, cu_blk,
                                         block_offsets, rope_mode, wsp, ws_bytes - (size_t)(wsp - (char *)ws), stream_)))
      return rc;
    if ((rc = move_heads(heads, o_out, o4.ptr, T, false, stream, "whole prompts: head un-padding launch"))) return rc;
    if (lse_out) {
      hipError_t e = ba::launch_pad_lse(lse_out, lse4, T, heads->n_kv_heads, G, kPadGroup, false, stream);
      if (e != hipSuccess) return device_fail(e, "whole prompts: log-sum-exp un-padding launch");
    }
    return BA_OK;
  }
  if ((max_len + 1) * widest >= 0x40000000 || max_len * G > 0x3fffffff)
    return fail(BA_ERR_UNSUPPORTED, "whole-prompt attention: a block of %lld tokens at these strides is too long",
                (long long)max_len);

  ba::RopeTable rt;
  build_rope_table(heads, &rt);
  ba_tensor k_use = *k;
  float *q_table = nullptr;
  if (rope_mode == BA_ROPE_APPLY) {
    const size_t need =
        ba_block_attention_prompts_workspace_bytes(heads, n_prompts, cu_blk, block_offsets, rope_mode, k_rot_out != nullptr);
    if (!ws || ws_bytes < need || ((uintptr_t)ws & 255))
      return fail(BA_ERR_WORKSPACE, "whole prompts: 256-byte aligned workspace of %zu bytes needed, %zu given", need,
                  ws_bytes);
    char *wsp = (char *)ws;
    if (k_rot_out) {
      k_use = *k_rot_out;
    } else {
      k_use.ptr = wsp;
      k_use.stride_head = D;
      k_use.stride_tok = (int64_t)heads->n_kv_heads * D;
      k_use.dtype = BA_DTYPE_BF16;
      wsp += align256((size_t)T * heads->n_kv_heads * D * 2);
    }
    q_table = (float *)wsp;
    // positions count from each prompt's first token: one segment per prompt
    std::vector<int32_t> starts(n_prompts + 1);
    for (int n = 0; n <= n_prompts; ++n) starts[n] = block_offsets[cu_blk[n]];
    for (int n0 = 0; n0 < n_prompts; n0 += ba::kRopeMaxSegs) {
      const int n = std::min(ba::kRopeMaxSegs, n_prompts - n0);
      if ((rc = run_rope_prepass(heads, rt, q, nullptr, k, &k_use, n, starts.data() + n0, nullptr, stream, nullptr,
                                 nullptr, nullptr, 0, q_table)))
        return rc;
    }
  }

  ba::AttnParams ap;
  memset(&ap, 0, sizeof(ap));
  ap.q = (const uint16_t *)q->ptr;
  ap.q_st = q->stride_tok;
  ap.q_sh = q->stride_head;
  ap.q_table = q_table;
  ap.kf = (const uint16_t *)k_use.ptr;
  ap.kf_st = k_use.stride_tok;
  ap.kf_sh = k_use.stride_head;
  ap.vf = (const uint16_t *)v->ptr;
  ap.vf_st = v->stride_tok;
  ap.vf_sh = v->stride_head;
  ap.kc = ap.kf;
  ap.kc_st = ap.kf_st;
  ap.kc_sh = ap.kf_sh;
  ap.vc = ap.vf;
  ap.vc_st = ap.vf_st;
  ap.vc_sh = ap.vf_sh;
  ap.o = (uint16_t *)o_out->ptr;
  ap.o_st = o_out->stride_tok;
  ap.o_sh = o_out->stride_head;
  ap.lse = lse_out;
  ap.n_q_heads = heads->n_q_heads;
  ap.n_kv_heads = heads->n_kv_heads;
  ap.group = G;
  ap.group_div = ba::make_fast_div((uint32_t)G);
  ap.head_dim = D;
  ap.scale_log2e = scale_log2e(heads);
  ap.q_ready = 0;
  ap.rope_layout = heads->rope_layout;
  ap.n_splits = 1;

  // Blocks go to the kernel longest key range first (see the planner).
  std::vector<ba::PromptBlock> blks = ba::list_prompt_blocks(n_prompts, cu_blk, block_offsets);
  ba::sort_by_key_range(&blks);
  const int n_live = (int)blks.size();

  for (int b0 = 0; b0 < n_live; b0 += ba::kEncMaxBlocks) {
    const int n = std::min(ba::kEncMaxBlocks, n_live - b0);
    ba::PromptMeta meta;
    const int64_t tiles = ba::build_prompt_meta(blks, (size_t)b0, n, G, &meta);
    if (tiles < 0) return fail(BA_ERR_INVALID_ARG, "too many row tiles in one call");
    if (tiles == 0) continue;
    ap.total_tiles = (int32_t)tiles;
    ap.tiles_div = ba::make_fast_div((uint32_t)tiles);
    hipError_t e;
    {
      ProfileScope ps(BA_PROFILE_ATTENTION, stream);
      e = ba::launch_attn_prompt_short(ap, meta, stream);
    }
    if (e != hipSuccess) return device_fail(e, "whole-prompt attention launch");
  }
  return BA_OK;
}

// ------------------------------------------------------------------------------------------
size_t ba_block_attention_prompts_backward_workspace_bytes(const ba_heads *heads, int32_t n_prompts,
                                                           const int32_t *cu_blk, const int32_t *block_offsets) {
  if (check_heads(heads, true) != BA_OK || check_prompt_blocks(n_prompts, cu_blk, block_offsets) != BA_OK) return 0;
  const size_t T = (size_t)block_offsets[cu_blk[n_prompts]];
  const size_t D = heads->head_dim, hkv = heads->n_kv_heads;
  size_t hq = heads->n_q_heads, pad_bytes = 0;
  if (hq / hkv < (size_t)kPadGroup) {  // padded q, o, d_out and dq, padded log-sum-exps; the rest for groups of four
    pad_bytes = 4 * padded_rows_bytes(heads, T) + padded_lse_bytes(heads, T);
    hq = hkv * kPadGroup;
  }
  // rotated scaled q, rotated k, the table of rotation factors, (log-sum-exp, delta) per row (+ padding)
  return pad_bytes + align256(T * hq * D * 2) + align256(T * hkv * D * 2) + align256(T * D * 4) + align256(T * hq * 8 + 16);
}

int32_t ba_block_attention_prompts_backward(const ba_heads *heads, const ba_tensor *q, const ba_tensor *k,
                                            const ba_tensor *v, const ba_tensor *o, const float *lse,
                                            const ba_tensor *d_out, const ba_tensor *dq_out,
                                            const ba_tensor *dk_out, const ba_tensor *dv_out, int32_t n_prompts,
                                            const int32_t *cu_blk, const int32_t *block_offsets, void *ws,
                                            size_t ws_bytes, void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  int32_t rc;
  if ((rc = check_heads(heads, true))) return rc;
  if ((rc = check_prompt_blocks(n_prompts, cu_blk, block_offsets))) return rc;
  const int n_blocks = cu_blk[n_prompts];
  const int D = heads->head_dim, hq = heads->n_q_heads, hkv = heads->n_kv_heads;
  if ((rc = check_tensor(q, "q", false, D, hq))) return rc;
  if ((rc = check_tensor(k, "k", false, D, hkv))) return rc;
  if ((rc = check_tensor(v, "v", false, D, hkv))) return rc;
  if ((rc = check_tensor(o, "o", false, D, hq))) return rc;
  if ((rc = check_tensor(d_out, "d_out", false, D, hq))) return rc;
  if ((rc = check_tensor(dq_out, "dq_out", false, D, hq))) return rc;
  if ((rc = check_tensor(dk_out, "dk_out", false, D, hkv))) return rc;
  if ((rc = check_tensor(dv_out, "dv_out", false, D, hkv))) return rc;
  if (!lse || ((uintptr_t)lse & 3)) return fail(BA_ERR_INVALID_ARG, "lse: null or misaligned");
  const int64_t T = block_offsets[n_blocks];
  const int G = hq / hkv;
  if (T == 0) return BA_OK;
  int64_t max_len = 0;
  for (int b = 0; b < n_blocks; ++b) max_len = std::max<int64_t>(max_len, (int64_t)block_offsets[b + 1] - block_offsets[b]);
  const int64_t widest =
      std::max(std::max((int64_t)hq * D, std::max(std::max(d_out->stride_tok, o->stride_tok), dq_out->stride_tok)),
               (int64_t)G * std::max((int64_t)D, std::max(std::max(d_out->stride_head, o->stride_head), dq_out->stride_head)));
  const size_t need = ba_block_attention_prompts_backward_workspace_bytes(heads, n_prompts, cu_blk, block_offsets);
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 255))
    return fail(BA_ERR_WORKSPACE, "whole prompts, backward: 256-byte aligned workspace of %zu bytes needed, %zu given",
                need, ws_bytes);
  if (G < kPadGroup) {
    // run as groups of four (see head_pad.hip): the phantom heads' output gradient is zero, so they add
    // nothing to dk and dv, which the padded call writes straight to the caller's tensors
    const ba_heads h4 = padded_heads(heads);
    char *wp = (char *)ws;
    const ba_tensor q4 = padded_tensor(wp, heads);
    wp += padded_rows_bytes(heads, (size_t)T);
    const ba_tensor o4 = padded_tensor(wp, heads);
    wp += padded_rows_bytes(heads, (size_t)T);
    const ba_tensor do4 = padded_tensor(wp, heads);
    wp += padded_rows_bytes(heads, (size_t)T);
    const ba_tensor dq4 = padded_tensor(wp, heads);
    wp += padded_rows_bytes(heads, (size_t)T);
    float *lse4 = (float *)wp;
    wp += padded_lse_bytes(heads, (size_t)T);
    if ((rc = move_heads(heads, q, q4.ptr, T, true, stream, "backward: head padding launch"))) return rc;
    if ((rc = move_heads(heads, o, o4.ptr, T, true, stream, "backward: head padding launch"))) return rc;
    if ((rc = move_heads(heads, d_out, do4.ptr, T, true, stream, "backward: head padding launch"))) return rc;
    hipError_t pe = ba::launch_pad_lse(const_cast<float *>(lse), lse4, T, hkv, G, kPadGroup, true, stream);
    if (pe != hipSuccess) return device_fail(pe, "backward: log-sum-exp padding launch");
    if ((rc = ba_block_attention_prompts_backward(&h4, &q4, k, v, &o4, lse4, &do4, &dq4, dk_out, dv_out, n_prompts, cu_blk,
                                                  block_offsets, wp, ws_bytes - (size_t)(wp - (char *)ws), stream_)))
      return rc;
    return move_heads(heads, dq_out, dq4.ptr, T, false, stream, "backward: head un-padding launch");
  }
  if ((max_len + 1) * widest >= 0x40000000 || max_len * G > 0x3fffffff)
    return fail(BA_ERR_UNSUPPORTED, "whole-prompt attention: a block of %lld tokens at these strides is too long",
                (long long)max_len);
  char *wsp = (char *)ws;
  uint16_t *q_rot = (uint16_t *)wsp;
  wsp += align256((size_t)T * hq * D * 2);
  ba_tensor k_rot;
  k_rot.ptr = wsp;
  k_rot.stride_head = D;
  k_rot.stride_tok = (int64_t)hkv * D;
  k_rot.dtype = BA_DTYPE_BF16;
  wsp += align256((size_t)T * hkv * D * 2);
  float *q_table = (float *)wsp;
  wsp += align256((size_t)T * D * 4);
  float2 *ld = (float2 *)wsp;

  ba::RopeTable rt;
  build_rope_table(heads, &rt);
  // positions count from each prompt's first token: one segment per prompt
  std::vector<int32_t> starts(n_prompts + 1);
  for (int n = 0; n <= n_prompts; ++n) starts[n] = block_offsets[cu_blk[n]];
  for (int n0 = 0; n0 < n_prompts; n0 += ba::kRopeMaxSegs) {
    const int n = std::min(ba::kRopeMaxSegs, n_prompts - n0);
    if ((rc = run_rope_prepass(heads, rt, q, q_rot, k, &k_rot, n, starts.data() + n0, nullptr, stream, nullptr, nullptr,
                               nullptr, 0, q_table, true)))
      return rc;
  }

  ba::BwdParams bp;
  memset(&bp, 0, sizeof(bp));
  bp.dout = (const uint16_t *)d_out->ptr;
  bp.do_st = d_out->stride_tok;
  bp.do_sh = d_out->stride_head;
  bp.o = (const uint16_t *)o->ptr;
  bp.o_st = o->stride_tok;
  bp.o_sh = o->stride_head;
  bp.lse = lse;
  bp.ld = ld;
  bp.T = T;
  bp.dq = (uint16_t *)dq_out->ptr;
  bp.dq_st = dq_out->stride_tok;
  bp.dq_sh = dq_out->stride_head;
  bp.dk = (uint16_t *)dk_out->ptr;
  bp.dk_st = dk_out->stride_tok;
  bp.dk_sh = dk_out->stride_head;
  bp.dv = (uint16_t *)dv_out->ptr;
  bp.dv_st = dv_out->stride_tok;
  bp.dv_sh = dv_out->stride_head;
  bp.scale = heads->softmax_scale > 0.f ? heads->softmax_scale : 1.0f / sqrtf((float)D);
  hipError_t e;

  ba::AttnParams ap;
  memset(&ap, 0, sizeof(ap));
  ap.q = q_rot;
  ap.q_st = (int64_t)hq * D;
  ap.q_sh = D;
  ap.kf = (const uint16_t *)k_rot.ptr;
  ap.kf_st = k_rot.stride_tok;
  ap.kf_sh = k_rot.stride_head;
  ap.vf = (const uint16_t *)v->ptr;
  ap.vf_st = v->stride_tok;
  ap.vf_sh = v->stride_head;
  ap.q_table = q_table;
  ap.scale_log2e = scale_log2e(heads);
  ap.rope_layout = heads->rope_layout;
  ap.n_q_heads = hq;
  ap.n_kv_heads = hkv;
  ap.group = G;
  ap.group_div = ba::make_fast_div((uint32_t)G);
  ap.head_dim = D;
  ap.n_splits = 1;

  const std::vector<ba::PromptBlock> blks = ba::list_prompt_blocks(n_prompts, cu_blk, block_offsets);
  typedef ba::PromptBlock Blk;
  // dq: query rows own the sums; longest key range first
  std::vector<Blk> by_q = blks;
  ba::sort_by_key_range(&by_q);
  for (size_t b0 = 0; b0 < by_q.size(); b0 += ba::kEncMaxBlocks) {
    const int n = (int)std::min<size_t>(ba::kEncMaxBlocks, by_q.size() - b0);
    ba::PromptMeta meta;
    const int64_t tiles = ba::build_prompt_meta(by_q, b0, n, G, &meta);
    if (tiles < 0) return fail(BA_ERR_INVALID_ARG, "too many row tiles in one call");
    if (tiles == 0) continue;
    ap.total_tiles = (int32_t)tiles;
    ap.tiles_div = ba::make_fast_div((uint32_t)tiles);
    {
      ProfileScope ps(BA_PROFILE_ATTENTION, stream);
      e = ba::launch_bwd_dq(ap, meta, bp, stream);
    }
    if (e != hipSuccess) return device_fail(e, "backward: dq launch");
  }
  // dk, dv: keys own the sums; most query rows first
  std::vector<Blk> by_k = blks;
  std::stable_sort(by_k.begin(), by_k.end(),
                   [](const Blk &a, const Blk &b) { return a.len + a.fin_len > b.len + b.fin_len; });
  for (size_t b0 = 0; b0 < by_k.size(); b0 += ba::kEncMaxBlocks) {
    const int n = (int)std::min<size_t>(ba::kEncMaxBlocks, by_k.size() - b0);
    ba::BwdKvMeta meta;
    memset(&meta, 0, sizeof(meta));
    meta.n = n;
    int64_t tiles = 0;
    for (int i = 0; i < n; ++i) {
      meta.start[i] = by_k[b0 + i].start;
      meta.len[i] = by_k[b0 + i].len;
      meta.fin_start[i] = by_k[b0 + i].fin_start;
      meta.fin_len[i] = by_k[b0 + i].fin_len;
      meta.tile_start[i] = (int32_t)tiles;
      tiles += ((int64_t)by_k[b0 + i].len + ba::kShortTileRows - 1) / ba::kShortTileRows;
    }
    meta.tile_start[n] = (int32_t)tiles;
    if (tiles > 0x3fffffff) return fail(BA_ERR_INVALID_ARG, "too many row tiles in one call");
    if (tiles == 0) continue;
    ap.total_tiles = (int32_t)tiles;
    ap.tiles_div = ba::make_fast_div((uint32_t)tiles);
    {
      ProfileScope ps(BA_PROFILE_ATTENTION, stream);
      e = ba::launch_bwd_dkv(ap, meta, bp, stream);
    }
    if (e != hipSuccess) return device_fail(e, "backward: dk/dv launch");
  }
  return BA_OK;
}

}  // extern "C"
