// C boundary of the Block-attention library: validation of the device tensors, workspace layout
// and kernel launches.  The planning (host arrays, KV splits, tables of row tiles) is ba_plan.cpp's.
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

namespace {

using ba::align256;
using ba::check_heads;
using ba::check_offsets;
using ba::check_prompt_blocks;
using ba::fail;
using ba::FinalPlan;
using ba::BlocksPlan;

int32_t device_fail(hipError_t e, const char *what) {
  return fail(BA_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

// ---- optional per-kernel timing (ba_profile_begin / ba_profile_end) ------------------------
struct Profiler {
  std::mutex mu;
  bool on = false;
  int max_records = 0;
  std::vector<hipEvent_t> start[BA_PROFILE_CLASSES], stop[BA_PROFILE_CLASSES];
} g_prof;

// Brackets one kernel launch with two events on its stream while profiling is on.
struct ProfileScope {
  hipStream_t stream;
  int cls;
  bool active = false;
  hipEvent_t stop_event = nullptr;  // this scope's own: another thread may open a scope of the class meanwhile
  ProfileScope(int cls_, hipStream_t s) : stream(s), cls(cls_) {
    std::lock_guard<std::mutex> lk(g_prof.mu);
    if (!g_prof.on || (int)g_prof.start[cls].size() >= g_prof.max_records) return;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return;
    if (hipEventCreate(&e1) != hipSuccess) {
      (void)hipEventDestroy(e0);
      return;
    }
    g_prof.start[cls].push_back(e0);
    g_prof.stop[cls].push_back(e1);
    (void)hipEventRecord(e0, stream);
    stop_event = e1;
    active = true;
  }
  ~ProfileScope() {
    if (!active) return;
    // (under the lock: ba_profile_end destroys the events, and must not do so between the
    // constructor and this record)
    std::lock_guard<std::mutex> lk(g_prof.mu);
    if (g_prof.on) (void)hipEventRecord(stop_event, stream);
  }
};

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

// Run the rotation kernel over a list of blocks, a launch per table-full of them.
template <typename Blocks>
int32_t run_reencode_t(ba::ReencParams p, const ba::RopeTable &rt, int n_blocks, const int32_t *src_off,
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
                         const int32_t *pos0, hipStream_t stream, const ba::RopeRots *rots = nullptr,
                         const ba::RopeRotsSmall *rots_small = nullptr, float *rot_dst = nullptr, int n_rot = 0,
                         float *q_table = nullptr, bool rows_too = false) {
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


// set by ba_measure_xcd_speed around its own final-block calls: where the workgroups leave their clock readings
thread_local unsigned long long *g_probe_clock = nullptr;

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

  for (int b0 = 0; b0 < n_blocks; b0 += ba::kEncMaxBlocks) {
    const int n = std::min(ba::kEncMaxBlocks, n_blocks - b0);
    ba::EncodeMeta meta[2];  // [0] main core, [1] short blocks
    int64_t tiles[2];
    if ((rc = ba::build_encode_metas(block_offsets, b0, n, G, short_max, meta, tiles))) return rc;
    if (tiles[0] + tiles[1] == 0) continue;
    if (rope_mode == BA_ROPE_APPLY) {  // local positions: every block starts at 0
      if ((rc = run_rope_prepass(heads, rt, q, nullptr, k, &k_use, n, meta[0].offs, nullptr, stream, nullptr, nullptr,
                                 nullptr, 0, q_table)))
        return rc;
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
  ap.wg_clock = g_probe_clock;  // (null unless ba_measure_xcd_speed is the caller)

  int64_t tile_base = 0;  // row tiles of the launches so far: the split partials are indexed by row tile
  for (int n0 = 0; n0 < n_prompts; n0 += ba::kFinMaxPrompts) {
    const int n = std::min(ba::kFinMaxPrompts, n_prompts - n0);
    ba::FinalMeta meta;
    const int64_t tiles = ba::build_final_meta(cu_q, cu_ctx, n0, n, G, &meta);
    ap.tile_base = (int32_t)tile_base;
    tile_base += tiles;
    ap.total_tiles = (int32_t)tiles;
    if ((rc = ba::plan_split_cuts(heads->xcd_speed, tiles, heads->n_kv_heads, pl.n_splits, pl.max_nt, num_cus(),
                                  ba::final_q_bytes_per_kv_head(heads, pl.lq_total), ap.split_cut, &ap.use_cuts, &ap.kv_group)))
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
                                            &ap.use_cuts, &ap.kv_group);
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

// ------------------------------------------------------------------------------------------
// Calibration: relative XCD speeds under the attention core's load (ba_heads.xcd_speed).
namespace {
constexpr int kProbeCtx = 31744, kProbeLq = 256, kProbeHq = 32, kProbeHkv = 8, kProbeD = 128;
constexpr int kProbeWarmRuns = 3, kProbeRuns = 4;  // launches to reach the steady clock, then launches that are read
constexpr int kProbeMaxWg = 4096;
ba_heads probe_heads() {
  ba_heads h;
  memset(&h, 0, sizeof(h));
  h.n_q_heads = kProbeHq;
  h.n_kv_heads = kProbeHkv;
  h.head_dim = kProbeD;
  h.rope_base = 500000.0;
  h.rope_layout = BA_ROPE_INTERLEAVED;
  return h;
}
struct ProbeLayout {
  size_t kv_bytes, q_bytes, kvf_bytes, clock_bytes, final_bytes;
  size_t total() const { return 2 * kv_bytes + 2 * q_bytes + 2 * kvf_bytes + clock_bytes + final_bytes; }
};
ProbeLayout probe_layout() {
  ProbeLayout l;
  l.kv_bytes = align256((size_t)kProbeCtx * kProbeHkv * kProbeD * 2);
  l.q_bytes = align256((size_t)kProbeLq * kProbeHq * kProbeD * 2);
  l.kvf_bytes = align256((size_t)kProbeLq * kProbeHkv * kProbeD * 2);
  l.clock_bytes = align256((size_t)kProbeMaxWg * ba::kProbeRecord * sizeof(unsigned long long) * kProbeRuns);
  const ba_heads h = probe_heads();
  const int32_t cu_q[2] = {0, kProbeLq}, cu_ctx[2] = {0, kProbeCtx};
  l.final_bytes = align256(ba_final_block_attention_workspace_bytes(&h, 1, cu_q, cu_ctx, BA_ROPE_NONE, 0));
  return l;
}
}  // namespace

extern "C" size_t ba_measure_xcd_speed_workspace_bytes(void) { return probe_layout().total(); }

namespace {
// Runs the probe launches and reads the workgroups' records back: kProbeRuns launches' worth, one
// after the other in *rec (the clocks of the XCDs drift by a few per cent from launch to launch, so
// one launch alone is a noisy sample).  Empty: the launch has a shape there is nothing to learn from.
// Synchronises the stream.
int32_t run_probe(void *ws, size_t ws_bytes, void *stream_, const float *xcd_speed, std::vector<unsigned long long> *rec,
                  int64_t *n_wg_out) {
  hipStream_t stream = (hipStream_t)stream_;
  rec->clear();
  *n_wg_out = 0;
  const ProbeLayout l = probe_layout();
  if (!ws || ws_bytes < l.total() || ((uintptr_t)ws & 255))
    return fail(BA_ERR_WORKSPACE, "final-block probe: 256-byte aligned workspace of %zu bytes needed, %zu given", l.total(),
                ws_bytes);
  char *wp = (char *)ws;
  ba_heads h = probe_heads();
  h.xcd_speed = xcd_speed;
  auto tensor = [&](size_t bytes, int heads_n) {
    ba_tensor t;
    t.ptr = wp;
    t.stride_head = kProbeD;
    t.stride_tok = (int64_t)heads_n * kProbeD;
    t.dtype = BA_DTYPE_BF16;
    wp += bytes;
    return t;
  };
  const ba_tensor kc = tensor(l.kv_bytes, kProbeHkv), vc = tensor(l.kv_bytes, kProbeHkv);
  const ba_tensor q = tensor(l.q_bytes, kProbeHq), o = tensor(l.q_bytes, kProbeHq);
  const ba_tensor kf = tensor(l.kvf_bytes, kProbeHkv), vf = tensor(l.kvf_bytes, kProbeHkv);
  unsigned long long *clk = (unsigned long long *)wp;
  wp += l.clock_bytes;
  // keys, values and queries with the bit activity of real data (the clock a part sustains depends on it)
  hipError_t e = ba::launch_fill_random_bf16((uint16_t *)kc.ptr, (2 * l.kv_bytes + l.q_bytes) / 2, 0x9e3779b9u, stream);
  if (e == hipSuccess)
    e = ba::launch_fill_random_bf16((uint16_t *)kf.ptr, 2 * l.kvf_bytes / 2, 0x85ebca6bu, stream);
  if (e == hipSuccess) e = hipMemsetAsync(clk, 0, l.clock_bytes, stream);
  if (e != hipSuccess) return device_fail(e, "final-block probe: fill");
  const int32_t cu_q[2] = {0, kProbeLq}, cu_ctx[2] = {0, kProbeCtx};
  int32_t rc = BA_OK;
  ba::FinalPlan pl;
  if ((rc = ba::plan_final(&h, 1, cu_q, cu_ctx, BA_ROPE_NONE, false, num_cus(), &pl))) return rc;
  const int64_t n_wg = pl.total_tiles * kProbeHkv * pl.n_splits;
  const bool readable = n_wg >= ba::kNumXcds && n_wg <= kProbeMaxWg;
  const size_t per_run = (size_t)n_wg * ba::kProbeRecord;
  if (readable) rec->resize(per_run * kProbeRuns);
  // (back to back, as a caller's layers run: a pause between launches lets the clocks recover and
  // shows a faster part than the one that does the work; every measured launch has records of its own)
  for (int run = 0; run < kProbeWarmRuns + kProbeRuns && rc == BA_OK; ++run) {
    g_probe_clock = run >= kProbeWarmRuns && readable ? clk + per_run * (run - kProbeWarmRuns) : nullptr;
    rc = ba_final_block_attention(&h, &q, &kc, &vc, &kf, &vf, &o, nullptr, 1, cu_q, cu_ctx, nullptr, BA_ROPE_NONE, wp,
                                  l.final_bytes, stream_);
    g_probe_clock = nullptr;
  }
  if (rc) return rc;
  if ((e = hipStreamSynchronize(stream)) != hipSuccess) return device_fail(e, "final-block probe: synchronize");
  if (!readable) return BA_OK;
  if ((e = hipMemcpy(rec->data(), clk, rec->size() * sizeof(unsigned long long), hipMemcpyDeviceToHost)) != hipSuccess)
    return device_fail(e, "final-block probe: read-back");
  *n_wg_out = n_wg;
  return BA_OK;
}
}  // namespace

extern "C" int32_t ba_measure_xcd_speed(float speed_out[8], void *ws, size_t ws_bytes, void *stream_) {
  if (!speed_out) return fail(BA_ERR_INVALID_ARG, "speed_out: null");
  float speed[ba::kNumXcds];
  for (int x = 0; x < ba::kNumXcds; ++x) speed_out[x] = speed[x] = 1.0f;
  // Two passes: equal splits first, then splits sized by the first pass's figures, whose residual
  // corrects them.  What is measured is how long an XCD's workgroups take from entry to the end of
  // their walk (not its clock alone: cycles per tile differ between XCDs too, with the place of their
  // keys in memory and with the causal tiles of the last split); a split's share is scaled by
  // mean / own, which equalises those times where time is proportional to tiles.
  for (int pass = 0; pass < 2; ++pass) {
    std::vector<unsigned long long> rec;
    int64_t n_wg = 0;
    if (int32_t rc = run_probe(ws, ws_bytes, stream_, pass ? speed : nullptr, &rec, &n_wg)) return rc;
    if (n_wg == 0) return BA_OK;  // nothing to learn from such a launch: equal speeds
    double sum[ba::kNumXcds] = {0}, total = 0.0;
    int cnt[ba::kNumXcds] = {0};
    for (int64_t i = 0; i < n_wg * kProbeRuns; ++i) {
      const unsigned long long *r = &rec[(size_t)i * ba::kProbeRecord];
      const int x = ba::xcd_of_workgroup((unsigned)(i % n_wg));
      if ((int)r[0] != x || r[5] <= r[2]) return BA_OK;  // not the mapping the planner assumes: equal speeds
      sum[x] += (double)(r[5] - r[2]);
      ++cnt[x];
    }
    for (int x = 0; x < ba::kNumXcds; ++x) {
      if (!cnt[x]) return BA_OK;
      sum[x] /= cnt[x];
      total += sum[x];
    }
    double next[ba::kNumXcds], norm = 0.0;
    for (int x = 0; x < ba::kNumXcds; ++x) {
      next[x] = (double)speed[x] * (total / ba::kNumXcds) / sum[x];
      norm += next[x];
    }
    for (int x = 0; x < ba::kNumXcds; ++x) {
      const double v = next[x] * ba::kNumXcds / norm;
      if (!(v >= 0.5 && v <= 2.0)) return BA_OK;  // implausible: keep equal speeds
      speed[x] = (float)v;
    }
  }
  for (int x = 0; x < ba::kNumXcds; ++x) speed_out[x] = speed[x];
  return BA_OK;
}

extern "C" int32_t ba_diag_final_block_phases(double phases_us[BA_DIAG_PHASES], const float *xcd_speed, void *ws,
                                              size_t ws_bytes, void *stream_) {
  if (!phases_us) return fail(BA_ERR_INVALID_ARG, "phases_us: null");
  for (int i = 0; i < BA_DIAG_PHASES; ++i) phases_us[i] = 0.0;
  std::vector<unsigned long long> rec;
  int64_t n_wg = 0;
  if (int32_t rc = run_probe(ws, ws_bytes, stream_, xcd_speed, &rec, &n_wg)) return rc;
  if (n_wg == 0) return fail(BA_ERR_UNSUPPORTED, "final-block phases: this device's launch is not the shape the probe times");
  // means over the launches that were read; per launch: its own first entry and last store
  const double tick_us = 0.01;  // the real-time counter runs at 100 MHz
  for (int run = 0; run < kProbeRuns; ++run) {
    const unsigned long long *base = &rec[(size_t)run * n_wg * ba::kProbeRecord];
    unsigned long long first = ~0ull, last = 0;
    double longest_walk = 0.0;
    for (int64_t wg = 0; wg < n_wg; ++wg) {
      const unsigned long long *r = base + (size_t)wg * ba::kProbeRecord;
      if (!(r[2] <= r[3] && r[3] <= r[6] && r[6] <= r[7] && r[7] <= r[5] && r[5] <= r[8] && r[8] <= r[9]))
        return fail(BA_ERR_DEVICE, "final-block phases: workgroup %lld left marks out of order", (long long)wg);
      first = std::min(first, r[2]);
      last = std::max(last, r[9]);
      phases_us[0] += (double)(r[3] - r[2]);
      phases_us[1] += (double)(r[6] - r[3]);
      phases_us[2] += (double)(r[7] - r[6]);
      phases_us[3] += (double)(r[5] - r[7]);
      phases_us[4] += (double)(r[9] - r[5]);
      phases_us[5] += (double)(r[9] - r[2]);
      longest_walk = std::max(longest_walk, (double)(r[5] - r[7]));
    }
    phases_us[6] += (double)(last - first) * (double)n_wg;  // (scaled like the sums above)
    phases_us[7] += longest_walk * (double)n_wg;
  }
  for (int i = 0; i < BA_DIAG_PHASES; ++i) phases_us[i] *= tick_us / ((double)n_wg * kProbeRuns);
  return BA_OK;
}

// ------------------------------------------------------------------------------------------
// Diagnostic: the MFMA rate the device sustains on data-like operands (see diag.hip).
extern "C" size_t ba_diag_mfma_ceiling_workspace_bytes(void) { return align256(ba::diag_mfma_workspace_bytes(num_cus())); }

extern "C" int32_t ba_diag_mfma_ceiling(int32_t lds_reads_per_two_mfma, double *tflops, double *clock_ghz,
                                        double *pipe_busy, void *ws, size_t ws_bytes, void *stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (lds_reads_per_two_mfma < 0 || lds_reads_per_two_mfma > 2)
    return fail(BA_ERR_INVALID_ARG, "lds_reads_per_two_mfma: 0, 1 or 2");
  const int n_wg = num_cus(), iters = 6000, runs = 5;
  const size_t need = ba_diag_mfma_ceiling_workspace_bytes();
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 255))
    return fail(BA_ERR_WORKSPACE, "MFMA diagnostic: 256-byte aligned workspace of %zu bytes needed, %zu given", need, ws_bytes);
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return device_fail(e, "MFMA diagnostic: event");
  if ((e = hipEventCreate(&e1)) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return device_fail(e, "MFMA diagnostic: event");
  }
  e = ba::launch_mfma_ceiling(lds_reads_per_two_mfma, n_wg, iters, ws, 1u, stream);  // warm-up
  if (e == hipSuccess) e = hipEventRecord(e0, stream);
  for (int r = 0; r < runs && e == hipSuccess; ++r) e = ba::launch_mfma_ceiling(lds_reads_per_two_mfma, n_wg, iters, ws, 7u + r, stream);
  if (e == hipSuccess) e = hipEventRecord(e1, stream);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  std::vector<unsigned long long> clk((size_t)n_wg * 8 * 2);
  if (e == hipSuccess) e = hipMemcpy(clk.data(), ws, clk.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return device_fail(e, "MFMA diagnostic");
  // Per workgroup, the wave that ran longest: the two waves of a SIMD do not share its matrix pipe
  // evenly (one may issue most of its loop before the other), so a single wave's time understates
  // how long the pipe was in use.
  double cyc = 0.0, ticks = 0.0, cyc_longest = 0.0;
  for (int wg = 0; wg < n_wg; ++wg) {
    unsigned long long longest = 0;
    for (int w = 0; w < 8; ++w) {
      const unsigned long long c = clk[((size_t)wg * 8 + w) * 2];
      cyc += (double)c;
      ticks += (double)clk[((size_t)wg * 8 + w) * 2 + 1];
      longest = std::max(longest, c);
    }
    cyc_longest += (double)longest;
  }
  const double waves = (double)n_wg * 8, mfma_per_wave = (double)iters * 16;
  if (tflops) *tflops = runs * waves * mfma_per_wave * 32768.0 / (ms * 1e-3) / 1e12;
  if (clock_ghz) *clock_ghz = ticks > 0 ? cyc / (10.0 * ticks) : 0.0;
  // two waves share a SIMD's matrix pipe, an MFMA of this shape occupies it for 32 cycles
  if (pipe_busy) *pipe_busy = cyc_longest > 0 ? mfma_per_wave * 32.0 * 2.0 / (cyc_longest / n_wg) : 0.0;
  return BA_OK;
}
