// C boundary of the Block-attention library: the helpers its files share (checks of the device
// tensors, RoPE table, launches of the re-encode and RoPE pre-pass kernels, per-kernel timing) and
// the entry points of the three steps of the hot path: per-block encoding, position re-encoding,
// final-block attention (workspace and static-scratch forms).  Whole prompts are ba_api_prompts.hip's,
// the block-table route ba_api_cached.hip's, calibration and diagnostics ba_probe.hip's, and all
// planning (host arrays, KV splits, tables of row tiles) ba_plan.cpp's.
// Nothing in this file touches device memory itself or synchronises.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>
#include <vector>

#include "../../include/ba.h"
#include "ba_internal.h"
#include "ba_plan.h"
#include "ba_api_common.h"

namespace ba {
int32_t device_fail(hipError_t e, const char *what) {
  return fail(BA_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}
// Compute units of the current device, asked once (256 on MI355X, which is also the fallback
// when no device can be asked, e.g. a workspace query on a machine without a GPU).
int num_cus() {
  static std::once_flag once;
  static int n = 256;
  std::call_once(once, [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
  });
  return n;
}
// set by the probes around their own final-block calls: where the workgroups leave their clock readings
unsigned long long *&probe_clock() {
  thread_local unsigned long long *clock = nullptr;
  return clock;
}
}  // namespace ba

namespace ba {
namespace api {
Profiler g_prof;

// run_reencode_t below is this file's own
size_t elt_size(int32_t dtype) { return dtype == BA_DTYPE_F32 ? 4 : 2; }

int32_t check_tensor(const ba_tensor *t, const char *name, bool allow_f32, int32_t D, int32_t n_heads) {
  if (!t || !t->ptr) return fail(BA_ERR_INVALID_ARG, "%s: null tensor", name);
  if (t->dtype != BA_DTYPE_BF16 && !(allow_f32 && t->dtype == BA_DTYPE_F32))
    return fail(BA_ERR_UNSUPPORTED, "%s: dtype %d not supported here", name, t->dtype);
  const size_t es = elt_size(t->dtype);
  if (((uintptr_t)t->ptr & 15) || ((t->stride_tok * (int64_t)es) & 15) || ((t->stride_head * (int64_t)es) & 15))
    return fail(BA_ERR_ALIGNMENT, "%s: pointer and strides must be 16-byte aligned", name);
  if (t->stride_head < D || t->stride_tok < (int64_t)D)
    return fail(BA_ERR_INVALID_ARG, "%s: strides smaller than head_dim", name);
  if (t->stride_tok >= (1 << 24))  // tile fills address rows with 32-bit byte offsets
    return fail(BA_ERR_UNSUPPORTED, "%s: token stride of 2^24 elements or more", name);
  (void)n_heads;
  return BA_OK;
}

// theta_j / (2 pi) as a Q0.64 fraction, from extended-precision host arithmetic.
void build_rope_table(const ba_heads *h, ba::RopeTable *rt) {
  // (64 extended-precision powers cost tens of microseconds, more than the launch of a small call:
  // the table of the last (base, head_dim) is kept per thread)
  struct Memo {
    bool valid = false;
    double base = 0.0;
    int head_dim = 0;
    ba::RopeTable rt;
  };
  static thread_local Memo memo;
  if (!h->inv_freq && memo.valid && memo.base == h->rope_base && memo.head_dim == h->head_dim) {
    *rt = memo.rt;
    return;
  }
  const long double two_pi = 6.283185307179586476925286766559005768L;
  const int half = h->head_dim / 2;
  for (int j = 0; j < ba::kMaxFreq; ++j) rt->turns[j] = 0;
  for (int j = 0; j < half; ++j) {
    long double th = h->inv_freq ? (long double)h->inv_freq[j]
                                 : powl((long double)h->rope_base, -2.0L * j / (long double)h->head_dim);
    long double turns = th / two_pi;
    turns -= floorl(turns);  // whole turns per position do not change the angle
    const long double up = ldexpl(turns, 32);  // split so each half fits 32 bits exactly
    const uint64_t hi = (uint64_t)floorl(up);
    const uint64_t lo = (uint64_t)floorl(ldexpl(up - floorl(up), 32));
    rt->turns[j] = (hi << 32) | (lo & 0xffffffffull);
  }
  if (!h->inv_freq) {
    memo.valid = true;
    memo.base = h->rope_base;
    memo.head_dim = h->head_dim;
    memo.rt = *rt;
  }
}

float scale_log2e(const ba_heads *h) {
  const double s = h->softmax_scale > 0.f ? (double)h->softmax_scale : 1.0 / sqrt((double)h->head_dim);
  return (float)(s * 1.4426950408889634074);
}


// Run the rotation kernel over a list of blocks, a launch per table-full of them.
template <typename Blocks>
static int32_t run_reencode_t(ba::ReencParams p, const ba::RopeTable &rt, int n_blocks, const int32_t *src_off,
                       const int32_t *dst_off, const int32_t *len, const int32_t *pos_old,
                       const int32_t *pos_new, hipStream_t stream) {
  std::vector<Blocks> tab(1);  // (the large table is too big for the stack of a small thread)
  Blocks &blk = tab[0];
  for (int b0 = 0; b0 < n_blocks; b0 += Blocks::kBlocks) {
    memset(&blk, 0, sizeof(blk));
    const int n = std::min(Blocks::kBlocks, n_blocks - b0);
    int filled = 0, max_len = 0;
    for (int i = 0; i < n; ++i) {
      const int b = b0 + i;
      if (len[b] == 0) continue;
      blk.src_off[filled] = src_off[b];
      blk.dst_off[filled] = dst_off[b];
      blk.len[filled] = len[b];
      blk.pos_old[filled] = pos_old ? pos_old[b] : 0;
      blk.pos_new[filled] = pos_new ? pos_new[b] : dst_off[b];
      max_len = std::max(max_len, len[b]);
      ++filled;
    }
    if (!filled) continue;
    blk.n = filled;
    p.max_len = max_len;
    // few tokens: one head per thread (more workgroups, shorter dependent chains);
    // many tokens: all heads in one thread (sin/cos computed once per token)
    int64_t tokens = 0;
    for (int i = 0; i < filled; ++i) tokens += blk.len[i];
    tokens *= p.n_layers;
    p.heads_per_thread = tokens >= 65536 ? p.n_kv_heads : (tokens >= 8192 ? std::min(p.n_kv_heads, 4) : 1);
    p.n_head_groups = (p.n_kv_heads + p.heads_per_thread - 1) / p.heads_per_thread;
    hipError_t e;
    {
      ProfileScope ps(BA_PROFILE_REENCODE, stream);
      e = ba::launch_reencode(p, blk, rt, stream);
    }
    if (e != hipSuccess) return device_fail(e, "re-encode launch");
  }
  return BA_OK;
}

int32_t run_reencode(ba::ReencParams p, const ba::RopeTable &rt, int n_blocks, const int32_t *src_off,
                     const int32_t *dst_off, const int32_t *len, const int32_t *pos_old,
                     const int32_t *pos_new, hipStream_t stream) {
  if (n_blocks > ba::kReencMaxBlocks)
    return run_reencode_t<ba::ReencBlocksLarge>(p, rt, n_blocks, src_off, dst_off, len, pos_old, pos_new, stream);
  return run_reencode_t<ba::ReencBlocks>(p, rt, n_blocks, src_off, dst_off, len, pos_old, pos_new, stream);
}

// Rotate fresh Q (into q_rot, packed, pre-scaled) and fresh K (into k_rot) for segments
// [seg0, seg0 + n) given by start offsets and first positions.
int32_t run_rope_prepass(const ba_heads *h, const ba::RopeTable &rt, const ba_tensor *q, uint16_t *q_rot,
                         const ba_tensor *k, const ba_tensor *k_rot, int n, const int32_t *start,
                         const int32_t *pos0, hipStream_t stream, const ba::RopeRots *rots,
                         const ba::RopeRotsSmall *rots_small, float *rot_dst, int n_rot, float *q_table, bool rows_too,
                         int table_rows) {
  const int64_t tokens = (int64_t)start[n] - start[0];
  if (tokens <= 0) return BA_OK;
  ba::RopePrepassParams p;
  memset(&p, 0, sizeof(p));
  const int D = h->head_dim;
  p.q_src = (const uint16_t *)q->ptr;
  p.q_dst = q_rot;
  p.q_st = q->stride_tok;
  p.q_sh = q->stride_head;
  p.qd_st = (int64_t)h->n_q_heads * D;
  p.qd_sh = D;
  p.k_src = (const uint16_t *)k->ptr;
  p.k_dst = (uint16_t *)k_rot->ptr;
  p.k_st = k->stride_tok;
  p.k_sh = k->stride_head;
  p.kd_st = k_rot->stride_tok;
  p.kd_sh = k_rot->stride_head;
  p.q_scale = scale_log2e(h);
  p.n_q_heads = h->n_q_heads;
  p.n_kv_heads = h->n_kv_heads;
  p.head_dim = D;
  p.layout = h->rope_layout;
  // few tokens: one head per thread (more, shorter threads); many: sin/cos shared by several heads
  p.heads_per_thread = tokens >= 16384 ? 8 : (tokens >= 2048 ? 2 : 1);
  p.do_q = q_table ? (rows_too ? 3 : 2) : 1;  // a table of factors for the attention core, rotated rows, or both
  p.q_table = q_table;
  if (table_rows > 0) {  // the table by position (every segment starts at position 0), no rotated rows
    p.do_q = 4;
    p.table_rows = table_rows;
  } else if (table_rows < 0) {  // keys only: the table of this call is already written
    p.do_q = 0;
  }
  p.do_k = 1;
  p.rot_dst = rot_dst;
  p.n_rot = n_rot;
  auto fill_and_launch = [&](auto &segs) {
    memset(&segs, 0, sizeof(segs));
    segs.n = n;
    for (int i = 0; i < n; ++i) {
      segs.start[i] = start[i];
      segs.pos0[i] = pos0 ? pos0[i] : 0;
    }
    segs.start[n] = start[n];
    ProfileScope ps(BA_PROFILE_REENCODE, stream);
    return ba::launch_rope_prepass(p, segs, rots, rots_small, rt, stream);
  };
  hipError_t e;
  if (n <= ba::kRopeSmallSegs) {
    ba::RopeSegsSmall segs;
    e = fill_and_launch(segs);
  } else {
    ba::RopeSegs segs;
    e = fill_and_launch(segs);
  }
  if (e != hipSuccess) return device_fail(e, "RoPE pre-pass launch");
  return BA_OK;
}



}  // namespace api
}  // namespace ba

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

extern "C" {

int32_t ba_version(void) { return 100; }

const char *ba_status_string(int32_t status) {
  switch (status) {
    case BA_OK: return "BA_OK";
    case BA_ERR_INVALID_ARG: return "BA_ERR_INVALID_ARG";
    case BA_ERR_UNSUPPORTED: return "BA_ERR_UNSUPPORTED";
    case BA_ERR_ALIGNMENT: return "BA_ERR_ALIGNMENT";
    case BA_ERR_WORKSPACE: return "BA_ERR_WORKSPACE";
    case BA_ERR_DEVICE: return "BA_ERR_DEVICE";
    default: return "BA_ERR_UNKNOWN";
  }
}

int32_t ba_profile_begin(int32_t max_records) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  if (g_prof.on) return fail(BA_ERR_INVALID_ARG, "profiling is already on");
  if (max_records < 1 || max_records > (1 << 20)) return fail(BA_ERR_INVALID_ARG, "max_records out of range");
  g_prof.on = true;
  g_prof.max_records = max_records;
  return BA_OK;
}

int32_t ba_profile_end(double *ms_sum, int32_t *launches) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  if (!g_prof.on) return fail(BA_ERR_INVALID_ARG, "profiling is not on");
  g_prof.on = false;
  int32_t rc = BA_OK;
  for (int c = 0; c < BA_PROFILE_CLASSES; ++c) {
    double sum = 0.0;
    int32_t n = 0;
    for (size_t i = 0; i < g_prof.start[c].size(); ++i) {
      float ms = 0.f;
      hipError_t e = hipEventSynchronize(g_prof.stop[c][i]);
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.start[c][i], g_prof.stop[c][i]);
      if (e == hipSuccess) {
        sum += ms;
        ++n;
      } else {
        rc = device_fail(e, "profile event");
      }
      (void)hipEventDestroy(g_prof.start[c][i]);
      (void)hipEventDestroy(g_prof.stop[c][i]);
    }
    g_prof.start[c].clear();
    g_prof.stop[c].clear();
    if (ms_sum) ms_sum[c] = sum;
    if (launches) launches[c] = n;
  }
  return rc;
}

// ------------------------------------------------------------------------------------------
size_t ba_encode_blocks_workspace_bytes(const ba_heads *heads, int32_t n_blocks,
                                        const int32_t *block_offsets, int32_t rope_mode,
                                        int32_t have_k_local_out) {
  if (check_heads(heads, true) != BA_OK || check_offsets(n_blocks, block_offsets) != BA_OK) return 0;
  if (rope_mode != BA_ROPE_APPLY) return 0;
  const size_t T = (size_t)block_offsets[n_blocks];
  const size_t k_bytes = have_k_local_out ? 0 : align256(T * heads->n_kv_heads * heads->head_dim * 2);
  return k_bytes + align256(T * heads->head_dim * 4);  // rotated K; scale * (cos, sin) per token and pair
}

int32_t ba_encode_blocks(const ba_heads *heads, const ba_tensor *q, const ba_tensor *k,
                         const ba_tensor *v, const ba_tensor *o_out, const ba_tensor *k_local_out,
                         int32_t n_blocks, const int32_t *block_offsets, int32_t rope_mode, void *ws,
                         size_t ws_bytes, void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  int32_t rc;
  if ((rc = check_heads(heads, true))) return rc;
  if ((rc = check_offsets(n_blocks, block_offsets))) return rc;
  const int D = heads->head_dim;
  if ((rc = check_tensor(q, "q", false, D, heads->n_q_heads))) return rc;
  if ((rc = check_tensor(k, "k", false, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(v, "v", false, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(o_out, "o_out", false, D, heads->n_q_heads))) return rc;
  if (rope_mode != BA_ROPE_NONE && rope_mode != BA_ROPE_APPLY)
    return fail(BA_ERR_INVALID_ARG, "rope_mode %d unknown", rope_mode);
  if (k_local_out) {
    if (rope_mode != BA_ROPE_APPLY)
      return fail(BA_ERR_INVALID_ARG, "k_local_out needs rope_mode BA_ROPE_APPLY");
    if ((rc = check_tensor(k_local_out, "k_local_out", false, D, heads->n_kv_heads))) return rc;
  }
  const int64_t T = block_offsets[n_blocks];
  const int G = heads->n_q_heads / heads->n_kv_heads;
  if (T == 0) return BA_OK;

  ba::RopeTable rt;
  build_rope_table(heads, &rt);

  // what the attention kernel reads: the caller's q and k (NONE), or with APPLY freshly rotated keys
  // (in k_local_out or the workspace) and the caller's q next to a table of rotation factors (in
  // the workspace) with which the kernel rotates its query rows itself: at this step's sizes a
  // round trip of the rotated queries through memory would cost more than the attention saves
  ba_tensor k_use = *k;
  float *q_table = nullptr;
  if (rope_mode == BA_ROPE_APPLY) {
    const size_t need = ba_encode_blocks_workspace_bytes(heads, n_blocks, block_offsets, rope_mode, k_local_out != nullptr);
    if (!ws || ws_bytes < need || ((uintptr_t)ws & 255))
      return fail(BA_ERR_WORKSPACE, "encode: 256-byte aligned workspace of %zu bytes needed, %zu given", need,
                  ws_bytes);
    char *wsp = (char *)ws;
    if (k_local_out) {
      k_use = *k_local_out;
    } else {
      k_use.ptr = wsp;
      k_use.stride_head = D;
      k_use.stride_tok = (int64_t)heads->n_kv_heads * D;
      k_use.dtype = BA_DTYPE_BF16;
      wsp += align256((size_t)T * heads->n_kv_heads * D * 2);
    }
    q_table = (float *)wsp;
  }

  ba::AttnParams ap;
  memset(&ap, 0, sizeof(ap));
  ap.q = (const uint16_t *)q->ptr;
  ap.q_st = q->stride_tok;
  ap.q_sh = q->stride_head;
  ap.q_table = q_table;
  ap.q_table_by_pos = 1;
  ap.kf = (const uint16_t *)k_use.ptr;
  ap.kf_st = k_use.stride_tok;
  ap.kf_sh = k_use.stride_head;
  ap.vf = (const uint16_t *)v->ptr;
  ap.vf_st = v->stride_tok;
  ap.vf_sh = v->stride_head;
  ap.kc = ap.kf;  // never dereferenced: no context segment
  ap.kc_st = ap.kf_st;
  ap.kc_sh = ap.kf_sh;
  ap.vc = ap.vf;
  ap.vc_st = ap.vf_st;
  ap.vc_sh = ap.vf_sh;
  ap.o = (uint16_t *)o_out->ptr;
  ap.o_st = o_out->stride_tok;
  ap.o_sh = o_out->stride_head;
  ap.n_q_heads = heads->n_q_heads;
  ap.n_kv_heads = heads->n_kv_heads;
  ap.group = G;
  ap.group_div = ba::make_fast_div((uint32_t)G);
  ap.head_dim = D;
  ap.scale_log2e = scale_log2e(heads);
  ap.q_ready = 0;
  ap.rope_layout = heads->rope_layout;
  ap.n_splits = 1;

  // short blocks take the schedule with small workgroups, several to a compute unit; longer ones the main core
  const int64_t widest = std::max(std::max(q->stride_tok, o_out->stride_tok),
                                  (int64_t)G * std::max(q->stride_head, o_out->stride_head));
  const int64_t short_max = ba::encode_short_max(G, widest);

  int64_t longest_block = 1;
  for (int b = 0; b < n_blocks; ++b) longest_block = std::max<int64_t>(longest_block, block_offsets[b + 1] - block_offsets[b]);
  bool table_written = false;
  for (int b0 = 0; b0 < n_blocks; b0 += ba::kEncMaxBlocks) {
    const int n = std::min(ba::kEncMaxBlocks, n_blocks - b0);
    ba::EncodeMeta meta[2];  // [0] main core, [1] short blocks
    int64_t tiles[2];
    if ((rc = ba::build_encode_metas(block_offsets, b0, n, G, short_max, meta, tiles))) return rc;
    if (tiles[0] + tiles[1] == 0) continue;
    if (rope_mode == BA_ROPE_APPLY) {
      // local positions: every block starts at 0, so one table of factors by position serves all blocks
      // (as many rows as the longest block has tokens; written by the first launch)
      if ((rc = run_rope_prepass(heads, rt, q, nullptr, k, &k_use, n, meta[0].offs, nullptr, stream, nullptr, nullptr,
                                 nullptr, 0, q_table, false, table_written ? -1 : (int)longest_block)))
        return rc;
      table_written = true;
    }
    for (int m = 1; m >= 0; --m) {
      if (tiles[m] == 0) continue;
      ap.total_tiles = (int32_t)tiles[m];
      ap.tiles_div = ba::make_fast_div((uint32_t)tiles[m]);
      hipError_t e;
      {
        ProfileScope ps(BA_PROFILE_ATTENTION, stream);
        e = m ? ba::launch_attn_encode_short(ap, meta[m], stream) : ba::launch_attn_encode(ap, meta[m], stream);
      }
      if (e != hipSuccess) return device_fail(e, "encode attention launch");
    }
  }
  return BA_OK;
}
// ------------------------------------------------------------------------------------------
int32_t ba_reencode_positions(const ba_heads *heads, const ba_tensor *k_src, const ba_tensor *k_dst,
                              int32_t n_layers, int64_t layer_stride_src, int64_t layer_stride_dst,
                              int32_t n_blocks, const int32_t *src_tok_off, const int32_t *dst_tok_off,
                              const int32_t *len, const int32_t *old_pos0, const int32_t *new_pos0,
                              int32_t mode, void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  int32_t rc;
  if ((rc = check_heads(heads, false))) return rc;
  const int D = heads->head_dim;
  if ((rc = check_tensor(k_src, "k_src", true, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(k_dst, "k_dst", true, D, heads->n_kv_heads))) return rc;
  if (k_src->dtype != k_dst->dtype) return fail(BA_ERR_UNSUPPORTED, "k_src and k_dst must share a dtype");
  if (mode != BA_REENC_SHIFT && mode != BA_REENC_ABSOLUTE)
    return fail(BA_ERR_INVALID_ARG, "mode %d unknown", mode);
  if (n_layers < 0 || n_blocks < 0) return fail(BA_ERR_INVALID_ARG, "negative layer or block count");
  if (n_blocks > 0 && (!src_tok_off || !dst_tok_off || !len))
    return fail(BA_ERR_INVALID_ARG, "src_tok_off / dst_tok_off / len: null");
  const size_t es = elt_size(k_src->dtype);
  if (n_layers > 1 && (((layer_stride_src * (int64_t)es) & 15) || ((layer_stride_dst * (int64_t)es) & 15)))
    return fail(BA_ERR_ALIGNMENT, "layer strides must be 16-byte aligned");
  if (n_layers > 65535) return fail(BA_ERR_UNSUPPORTED, "more than 65535 layers in one call");
  for (int b = 0; b < n_blocks; ++b)
    if (len[b] < 0 || src_tok_off[b] < 0 || dst_tok_off[b] < 0)
      return fail(BA_ERR_INVALID_ARG, "block %d: negative offset or length", b);

  // aliasing: either exactly in place, or destination spans disjoint from source spans
  const bool same_buf = k_src->ptr == k_dst->ptr;
  if (same_buf) {
    bool in_place = k_src->stride_tok == k_dst->stride_tok && k_src->stride_head == k_dst->stride_head &&
                    (n_layers <= 1 || layer_stride_src == layer_stride_dst);
    for (int b = 0; b < n_blocks && in_place; ++b) in_place = src_tok_off[b] == dst_tok_off[b];
    if (!in_place) return fail(BA_ERR_INVALID_ARG, "k_dst aliases k_src but is not exactly in place");
  } else {
    // token extents touched, per layer, in bytes from the base pointers
    int64_t src_hi = 0, dst_hi = 0;
    for (int b = 0; b < n_blocks; ++b) {
      src_hi = std::max<int64_t>(src_hi, (int64_t)src_tok_off[b] + len[b]);
      dst_hi = std::max<int64_t>(dst_hi, (int64_t)dst_tok_off[b] + len[b]);
    }
    // (up to the last element touched: the last token's last head, not a whole token stride beyond it,
    // or a view into a wider buffer would seem to reach into whatever is allocated behind that buffer)
    const int64_t last_head = (int64_t)(heads->n_kv_heads - 1);
    const int64_t src_span =
        ((n_layers - 1) * layer_stride_src + (src_hi - 1) * k_src->stride_tok + last_head * k_src->stride_head + D) * (int64_t)es;
    const int64_t dst_span =
        ((n_layers - 1) * layer_stride_dst + (dst_hi - 1) * k_dst->stride_tok + last_head * k_dst->stride_head + D) * (int64_t)es;
    const char *s0 = (const char *)k_src->ptr, *d0 = (const char *)k_dst->ptr;
    if (n_layers > 0 && src_hi > 0 && dst_hi > 0 && s0 < d0 + dst_span && d0 < s0 + src_span)
      return fail(BA_ERR_INVALID_ARG, "k_dst overlaps k_src without being exactly in place");
  }
  {
    // destination blocks must not overlap each other (in place as well: a token listed twice would
    // be rotated twice, or by two workgroups at once)
    std::vector<std::pair<int64_t, int64_t>> spans;
    for (int b = 0; b < n_blocks; ++b)
      if (len[b] > 0) spans.emplace_back(dst_tok_off[b], (int64_t)dst_tok_off[b] + len[b]);
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
      if (spans[i].first < spans[i - 1].second)
        return fail(BA_ERR_INVALID_ARG, "destination blocks overlap each other");
  }
  if (n_layers == 0 || n_blocks == 0) return BA_OK;

  ba::RopeTable rt;
  build_rope_table(heads, &rt);
  ba::ReencParams rp;
  memset(&rp, 0, sizeof(rp));
  rp.src = k_src->ptr;
  rp.dst = k_dst->ptr;
  rp.src_st = k_src->stride_tok;
  rp.src_sh = k_src->stride_head;
  rp.dst_st = k_dst->stride_tok;
  rp.dst_sh = k_dst->stride_head;
  rp.src_sl = layer_stride_src;
  rp.dst_sl = layer_stride_dst;
  rp.n_layers = n_layers;
  rp.n_kv_heads = heads->n_kv_heads;
  rp.head_dim = D;
  rp.dtype = k_src->dtype;
  rp.layout = heads->rope_layout;
  rp.mode = mode;
  rp.copy_from_layer = 0x7fffffff;
  return run_reencode(rp, rt, n_blocks, src_tok_off, dst_tok_off, len, old_pos0, new_pos0, stream);
}

// ------------------------------------------------------------------------------------------
size_t ba_final_block_attention_workspace_bytes(const ba_heads *heads, int32_t n_prompts,
                                                const int32_t *cu_q, const int32_t *cu_ctx,
                                                int32_t rope_mode, int32_t have_k_f_rot_out) {
  if (check_heads(heads, true) != BA_OK) return 0;
  FinalPlan pl;
  if (ba::plan_final(heads, n_prompts, cu_q, cu_ctx, rope_mode, have_k_f_rot_out != 0, num_cus(), &pl) != BA_OK) return 0;
  return pl.total();
}

int32_t ba_final_block_attention(const ba_heads *heads, const ba_tensor *q_f, const ba_tensor *k_ctx,
                                 const ba_tensor *v_ctx, const ba_tensor *k_f, const ba_tensor *v_f,
                                 const ba_tensor *o_out, const ba_tensor *k_f_rot_out, int32_t n_prompts,
                                 const int32_t *cu_q, const int32_t *cu_ctx, const int32_t *q_pos0,
                                 int32_t rope_mode, void *ws, size_t ws_bytes, void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  int32_t rc;
  if ((rc = check_heads(heads, true))) return rc;
  const int D = heads->head_dim;
  if (rope_mode != BA_ROPE_NONE && rope_mode != BA_ROPE_APPLY)
    return fail(BA_ERR_INVALID_ARG, "rope_mode %d unknown", rope_mode);
  FinalPlan pl;
  if ((rc = ba::plan_final(heads, n_prompts, cu_q, cu_ctx, rope_mode, k_f_rot_out != nullptr, num_cus(), &pl))) return rc;
  if (n_prompts == 0) return BA_OK;
  if ((rc = check_tensor(q_f, "q_f", false, D, heads->n_q_heads))) return rc;
  if ((rc = check_tensor(k_f, "k_f", false, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(v_f, "v_f", false, D, heads->n_kv_heads))) return rc;
  if ((rc = check_tensor(o_out, "o_out", false, D, heads->n_q_heads))) return rc;
  const bool any_ctx = cu_ctx[n_prompts] > cu_ctx[0];
  if (any_ctx) {
    if ((rc = check_tensor(k_ctx, "k_ctx", false, D, heads->n_kv_heads))) return rc;
    if ((rc = check_tensor(v_ctx, "v_ctx", false, D, heads->n_kv_heads))) return rc;
  }
  if (k_f_rot_out) {
    if (rope_mode != BA_ROPE_APPLY)
      return fail(BA_ERR_INVALID_ARG, "k_f_rot_out needs rope_mode BA_ROPE_APPLY");
    if ((rc = check_tensor(k_f_rot_out, "k_f_rot_out", false, D, heads->n_kv_heads))) return rc;
  }
  if (pl.total() > 0 && (!ws || ws_bytes < pl.total() || ((uintptr_t)ws & 255)))
    return fail(BA_ERR_WORKSPACE, "final block: 256-byte aligned workspace of %zu bytes needed, %zu given",
                pl.total(), ws_bytes);

  char *wsp = (char *)ws;
  void *kf_ws = wsp;
  uint16_t *q_ws = (uint16_t *)(wsp + align256(pl.kf_bytes));
  uint16_t *part_o = (uint16_t *)(wsp + align256(pl.kf_bytes) + align256(pl.q_bytes));
  float *part_ml = (float *)(wsp + align256(pl.kf_bytes) + align256(pl.q_bytes) + align256(pl.part_o_bytes));
  int32_t *part_idx = (int32_t *)((char *)part_ml + align256(pl.part_ml_bytes));

  ba::RopeTable rt;
  build_rope_table(heads, &rt);

  std::vector<int32_t> pos0(n_prompts), lens(n_prompts), starts(n_prompts), zero(n_prompts, 0);
  for (int n = 0; n < n_prompts; ++n) {
    pos0[n] = q_pos0 ? q_pos0[n] : cu_ctx[n + 1] - cu_ctx[n];
    lens[n] = cu_q[n + 1] - cu_q[n];
    starts[n] = cu_q[n];
  }

  ba_tensor kf_use = *k_f;
  if (rope_mode == BA_ROPE_APPLY) {
    if (k_f_rot_out) {
      kf_use = *k_f_rot_out;
    } else {
      kf_use.ptr = kf_ws;
      kf_use.stride_head = D;
      kf_use.stride_tok = (int64_t)heads->n_kv_heads * D;
    }
  }

  const int G = heads->n_q_heads / heads->n_kv_heads;
  ba::AttnParams ap;
  memset(&ap, 0, sizeof(ap));
  if (rope_mode == BA_ROPE_APPLY) {
    ap.q = q_ws;
    ap.q_st = (int64_t)heads->n_q_heads * D;
    ap.q_sh = D;
  } else {
    ap.q = (const uint16_t *)q_f->ptr;
    ap.q_st = q_f->stride_tok;
    ap.q_sh = q_f->stride_head;
  }
  ap.kf = (const uint16_t *)kf_use.ptr;
  ap.kf_st = kf_use.stride_tok;
  ap.kf_sh = kf_use.stride_head;
  ap.vf = (const uint16_t *)v_f->ptr;
  ap.vf_st = v_f->stride_tok;
  ap.vf_sh = v_f->stride_head;
  if (any_ctx) {
    ap.kc = (const uint16_t *)k_ctx->ptr;
    ap.kc_st = k_ctx->stride_tok;
    ap.kc_sh = k_ctx->stride_head;
    ap.vc = (const uint16_t *)v_ctx->ptr;
    ap.vc_st = v_ctx->stride_tok;
    ap.vc_sh = v_ctx->stride_head;
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
  ap.q_ready = rope_mode == BA_ROPE_APPLY;
  ap.rope_layout = heads->rope_layout;
  ap.n_splits = pl.n_splits;
  ap.wg_clock = ba::probe_clock();  // (null unless a probe of ba_probe.hip is the caller)

  int64_t tile_base = 0;  // row tiles of the launches so far: the split partials are indexed by row tile
  for (int n0 = 0; n0 < n_prompts; n0 += ba::kFinMaxPrompts) {
    const int n = std::min(ba::kFinMaxPrompts, n_prompts - n0);
    ba::FinalMeta meta;
    const int64_t tiles = ba::build_final_meta(cu_q, cu_ctx, n0, n, G, &meta);
    ap.tile_base = (int32_t)tile_base;
    tile_base += tiles;
    ap.total_tiles = (int32_t)tiles;
    if ((rc = ba::plan_split_cuts(heads->xcd_speed, tiles, heads->n_kv_heads, pl.n_splits, pl.max_nt, num_cus(),
                                  ba::final_q_bytes_per_kv_head(heads, pl.lq_total), ap.split_cut, &ap.use_cuts, &ap.kv_group,
                                  &ap.xcd_runs)))
      return rc;
    if (rope_mode == BA_ROPE_APPLY) {  // absolute positions of the final block's tokens
      if ((rc = run_rope_prepass(heads, rt, q_f, q_ws, k_f, &kf_use, n, meta.cu_q, pos0.data() + n0, stream)))
        return rc;
    }
    hipError_t e;
    {
      ProfileScope ps(BA_PROFILE_ATTENTION, stream);
      e = ba::launch_attn_final(ap, meta, stream);
    }
    if (e != hipSuccess) return device_fail(e, "final-block attention launch");
  }
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

// ------------------------------------------------------------------------------------------
// The allocation-free variant of ba_final_block_attention keeps its workspace (rotated final-block
// q and k, split partials) in this array.  The name is a host-side stand-in for the symbol: host
// code only ever uses the device address looked up per device below.
static __device__ __align__(256) unsigned char scratch[BA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (every GPU holds its own copy of the array).
int32_t scratch_address(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return device_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(BA_ERR_UNSUPPORTED, "device ordinal %d beyond %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return device_fail(e, "hipGetSymbolAddress(scratch)");
    if (!ptr || ((uintptr_t)ptr & 255)) return fail(BA_ERR_DEVICE, "static scratch: null or misaligned address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return BA_OK;
}
}  // namespace

extern "C" int32_t ba_final_block_attention_static(const ba_heads *heads, const ba_tensor *q_f, const ba_tensor *k_ctx,
                                        const ba_tensor *v_ctx, const ba_tensor *k_f, const ba_tensor *v_f,
                                        const ba_tensor *o_out, const ba_tensor *k_f_rot_out, int32_t n_prompts,
                                        const int32_t *cu_q, const int32_t *cu_ctx, const int32_t *q_pos0,
                                        int32_t rope_mode, void *stream_) {
  int32_t rc;
  if ((rc = check_heads(heads, true))) return rc;
  if (rope_mode != BA_ROPE_NONE && rope_mode != BA_ROPE_APPLY)
    return fail(BA_ERR_INVALID_ARG, "rope_mode %d unknown", rope_mode);
  FinalPlan pl;
  if ((rc = ba::plan_final(heads, n_prompts, cu_q, cu_ctx, rope_mode, k_f_rot_out != nullptr, num_cus(), &pl))) return rc;
  if (pl.total() > (size_t)BA_STATIC_SCRATCH_BYTES)
    return fail(BA_ERR_WORKSPACE, "final block (static scratch): this call needs %zu bytes of workspace, the array holds %zu",
                pl.total(), (size_t)BA_STATIC_SCRATCH_BYTES);
  void *ws = nullptr;
  if ((rc = scratch_address(&ws))) return rc;
  // Every byte of the workspace that a call reads it has written before (rotated rows by the RoPE
  // pre-pass, every split's partial of every row by the attention core), so nothing needs clearing.
  return ba_final_block_attention(heads, q_f, k_ctx, v_ctx, k_f, v_f, o_out, k_f_rot_out, n_prompts, cu_q, cu_ctx,
                                  q_pos0, rope_mode, ws, (size_t)BA_STATIC_SCRATCH_BYTES, stream_);
}
