// Host-side planning (see ba_plan.h) and the schedule queries of the C boundary.  No device code
// and no device calls in this file.
#include "ba_plan.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>

namespace ba {

namespace {
thread_local char g_err[512] = "";
}

int32_t fail(int32_t status, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return status;
}

const char *last_error() { return g_err; }

int32_t check_heads(const ba_heads *h, bool attention) {
  if (!h) return fail(BA_ERR_INVALID_ARG, "heads: null");
  if (h->head_dim != 64 && h->head_dim != 128)
    return fail(BA_ERR_UNSUPPORTED, "head_dim %d: only 64 and 128 are built", h->head_dim);
  if (h->n_kv_heads <= 0) return fail(BA_ERR_INVALID_ARG, "n_kv_heads must be positive");
  if (h->rope_layout != BA_ROPE_INTERLEAVED && h->rope_layout != BA_ROPE_HALF)
    return fail(BA_ERR_INVALID_ARG, "rope_layout %d unknown", h->rope_layout);
  if (!h->inv_freq && !(h->rope_base > 0.0)) return fail(BA_ERR_INVALID_ARG, "rope_base must be positive");
  if (attention) {
    if (h->n_q_heads <= 0 || h->n_q_heads % h->n_kv_heads)
      return fail(BA_ERR_INVALID_ARG, "n_q_heads must be a positive multiple of n_kv_heads");
    const int g = h->n_q_heads / h->n_kv_heads;
    if (h->q_to_kv)
      for (int i = 0; i < h->n_q_heads; ++i)
        if (h->q_to_kv[i] != i / g)
          return fail(BA_ERR_UNSUPPORTED, "q_to_kv: only the map h -> h / group is built");
  }
  return BA_OK;
}

int32_t check_offsets(int32_t n_blocks, const int32_t *offs) {
  if (n_blocks < 0 || !offs) return fail(BA_ERR_INVALID_ARG, "block_offsets: null or negative block count");
  if (offs[0] != 0) return fail(BA_ERR_INVALID_ARG, "block_offsets[0] must be 0");
  for (int b = 0; b < n_blocks; ++b)
    if (offs[b + 1] < offs[b]) return fail(BA_ERR_INVALID_ARG, "block_offsets must not decrease (block %d)", b);
  return BA_OK;
}

int32_t check_prompt_blocks(int32_t n_prompts, const int32_t *cu_blk, const int32_t *block_offsets) {
  if (n_prompts < 0 || !cu_blk) return fail(BA_ERR_INVALID_ARG, "cu_blk: null or negative prompt count");
  if (cu_blk[0] != 0) return fail(BA_ERR_INVALID_ARG, "cu_blk[0] must be 0");
  for (int n = 0; n < n_prompts; ++n)
    if (cu_blk[n + 1] <= cu_blk[n]) return fail(BA_ERR_INVALID_ARG, "prompt %d: at least one block needed", n);
  return check_offsets(cu_blk[n_prompts], block_offsets);
}

// One workgroup runs per compute unit, so a launch takes ceil(workgroups / CUs) rounds, each as long
// as one workgroup: a fixed part (prologue, output, worth about four key tiles) plus its share of the
// key tiles; every split also adds a little to the merge.  Take the cheapest count, never fewer than
// four key tiles per split.
int choose_splits(int64_t base_wgs, int max_tiles, int n_cu) {
  if (base_wgs <= 0) return 1;
  if (n_cu < 1) n_cu = 1;
  const int s_max = (int)std::min<int64_t>(32, std::max(1, max_tiles / 4));
  int best = 1;
  double best_cost = 0;
  for (int s = 1; s <= s_max; ++s) {
    const double rounds = (double)((base_wgs * s + n_cu - 1) / n_cu);
    const double cost = rounds * (4.0 + (max_tiles + s - 1) / s) + 0.25 * s;
    if (s == 1 || cost < best_cost) {
      best = s;
      best_cost = cost;
    }
  }
  return best;
}

int32_t plan_final(const ba_heads *h, int32_t n_prompts, const int32_t *cu_q, const int32_t *cu_ctx,
                   int32_t rope_mode, bool have_rot_out, int n_cu, FinalPlan *plan) {
  if (n_prompts < 0 || (n_prompts > 0 && (!cu_q || !cu_ctx)))
    return fail(BA_ERR_INVALID_ARG, "cu_q / cu_ctx: null or negative prompt count");
  const int G = h->n_q_heads / h->n_kv_heads;
  FinalPlan pl;
  if (n_prompts > 0 && cu_q[0] != 0) return fail(BA_ERR_INVALID_ARG, "cu_q[0] must be 0");
  if (n_prompts > 0 && cu_ctx[0] < 0) return fail(BA_ERR_INVALID_ARG, "cu_ctx[0] must not be negative");
  for (int n = 0; n < n_prompts; ++n) {
    const int64_t lq = (int64_t)cu_q[n + 1] - cu_q[n];
    const int64_t tc = (int64_t)cu_ctx[n + 1] - cu_ctx[n];
    if (lq < 1) return fail(BA_ERR_INVALID_ARG, "prompt %d: the final block needs at least one token", n);
    if (tc < 0) return fail(BA_ERR_INVALID_ARG, "prompt %d: cu_ctx decreases", n);
    if (lq * G > 0x3fffffff) return fail(BA_ERR_INVALID_ARG, "prompt %d: too many packed rows", n);
    pl.total_tiles += (lq * G + kTileRows - 1) / kTileRows;
    const int nt = (int)((tc + kTileKeys - 1) / kTileKeys + (lq + kTileKeys - 1) / kTileKeys);
    pl.max_nt = std::max(pl.max_nt, nt);
  }
  pl.lq_total = n_prompts > 0 ? cu_q[n_prompts] : 0;
  pl.n_splits = choose_splits(pl.total_tiles * h->n_kv_heads, pl.max_nt, n_cu);
  if (rope_mode == BA_ROPE_APPLY) {
    if (!have_rot_out) pl.kf_bytes = (size_t)pl.lq_total * h->n_kv_heads * h->head_dim * 2;
    pl.q_bytes = (size_t)pl.lq_total * h->n_q_heads * h->head_dim * 2;  // rotated, pre-scaled queries
  }
  if (pl.n_splits > 1) {
    const size_t rows = partial_rows(pl.total_tiles, h->n_kv_heads);
    pl.part_o_bytes = (size_t)pl.n_splits * rows * h->head_dim * 2;  // fp16
    pl.part_ml_bytes = (size_t)pl.n_splits * rows * 2 * 4;
    pl.part_idx_bytes = rows * 4;
  }
  *plan = pl;
  return BA_OK;
}

namespace {
// Cut lists of one candidate order of the work items, and how long its launch is expected to take,
// in tile periods of a workgroup: an XCD is done when its longest item is, or when its compute
// units have worked through all its items, whichever is later; before that it fetches the query
// rows of the KV heads it hosts (about a megabyte per microsecond and XCD, a tile period being 1.6).
double try_kv_group(const float *speed, int64_t tiles, int n_kv_heads, int n_splits, int kv_group, unsigned runs, int max_nt,
                    int n_cu, double q_bytes_per_kv_head, uint32_t cuts[kMaxCutHeads][33]) {
  const ItemOrder order = {(int)tiles, n_kv_heads, n_splits, kv_group};
  const unsigned n_wg = (unsigned)(tiles * n_kv_heads * n_splits);
  double longest[kNumXcds] = {0}, sum[kNumXcds] = {0};
  bool hosts[kNumXcds][kMaxCutHeads] = {};
  for (int h = 0; h < n_kv_heads; ++h) {
    double w[kMaxSplits], total = 0.0;
    for (int s = 0; s < n_splits; ++s) {
      double acc = 0.0;
      for (int64_t t = 0; t < tiles; ++t) acc += speed[xcd_of_work_item(item_id((int)t, h, s, order), n_wg, runs)];
      w[s] = acc / (double)tiles;
      total += w[s];
    }
    double acc = 0.0;
    for (int s = 0; s < n_splits; ++s) {
      cuts[h][s] = (uint32_t)(acc / total * 65536.0 + 0.5);
      acc += w[s];
    }
    for (int s = n_splits; s <= kMaxSplits; ++s) cuts[h][s] = 65536;
    for (int s = 0; s < n_splits; ++s) {
      const double item_tiles = (double)max_nt * (double)(cuts[h][s + 1] - cuts[h][s]) / 65536.0;
      for (int64_t t = 0; t < tiles; ++t) {
        const int x = xcd_of_work_item(item_id((int)t, h, s, order), n_wg, runs);
        longest[x] = std::max(longest[x], item_tiles);
        sum[x] += item_tiles;
        hosts[x][h] = true;
      }
    }
  }
  const double cu_per_xcd = std::max(1.0, (double)n_cu / kNumXcds);
  double worst = 0.0;
  for (int x = 0; x < kNumXcds; ++x) {
    int hosted = 0;
    for (int h = 0; h < n_kv_heads; ++h) hosted += hosts[x][h];
    const double fetch = hosted * q_bytes_per_kv_head / 1.0e6 / 1.6;
    worst = std::max(worst, std::max(longest[x], sum[x] / cu_per_xcd) / (double)speed[x] + fetch);
  }
  return worst;
}

// Which run of work items each XCD takes (work_item_of_workgroup) under groups of kv_group KV heads:
// the runs of one group of KV heads are neighbours, and only their XCDs can be balanced against each
// other, so the XCDs are dealt to the groups in order of speed, to and fro (fastest and slowest end
// up together), which brings the groups' mean speeds as close as a greedy deal gets them.  Identity
// when the runs do not line up with the groups.
unsigned deal_xcd_runs(const float *speed, int64_t tiles, int n_kv_heads, int n_splits, int kv_group) {
  const int64_t n_wg = tiles * n_kv_heads * n_splits;
  if (n_wg % kNumXcds || (kNumXcds * kv_group) % n_kv_heads) return kIdentityXcdRuns;
  const int per_group = kNumXcds * kv_group / n_kv_heads;  // runs (= XCDs) that share one group of KV heads
  if (per_group < 2 || per_group >= kNumXcds || kNumXcds % per_group) return kIdentityXcdRuns;
  const int n_groups = kNumXcds / per_group;
  int by_speed[kNumXcds];
  for (int x = 0; x < kNumXcds; ++x) by_speed[x] = x;
  std::stable_sort(by_speed, by_speed + kNumXcds, [&](int a, int b) { return speed[a] > speed[b]; });
  int taken[kNumXcds] = {0};
  unsigned runs = 0;
  for (int i = 0; i < kNumXcds; ++i) {
    const int pass = i / n_groups, pos = i % n_groups;
    const int group = (pass & 1) ? n_groups - 1 - pos : pos;
    runs |= (unsigned)(group * per_group + taken[group]++) << (4 * by_speed[i]);
  }
  return runs;
}
}  // namespace

int32_t plan_split_cuts(const float *xcd_speed, int64_t tiles, int n_kv_heads, int n_splits, int max_nt, int n_cu,
                        double q_bytes_per_kv_head, uint32_t cuts[kMaxCutHeads][33], int32_t *use, int32_t *kv_group,
                        uint32_t *xcd_runs) {
  *use = 0;
  *kv_group = kDefaultKvGroup;
  *xcd_runs = kIdentityXcdRuns;
  for (int h = 0; h < kMaxCutHeads; ++h)
    for (int s = 0; s <= kMaxSplits; ++s) cuts[h][s] = 0;
  if (!xcd_speed || n_splits <= 1 || tiles <= 0) return BA_OK;
  if (n_splits > kMaxSplits) return fail(BA_ERR_INVALID_ARG, "more than %d splits", kMaxSplits);
  for (int x = 0; x < kNumXcds; ++x)
    if (!(xcd_speed[x] >= 0.5f && xcd_speed[x] <= 2.0f))
      return fail(BA_ERR_INVALID_ARG, "xcd_speed[%d] = %g: relative speeds lie between 0.5 and 2", x, (double)xcd_speed[x]);
  if (n_kv_heads > kMaxCutHeads || tiles * n_kv_heads * n_splits > 0x7fffffff) return BA_OK;  // equal splits
  // The speed of (KV head, split) = the mean speed of the XCDs that run its row tiles (item_id,
  // xcd_of_work_item), and a KV head's key range is shared out in proportion to its splits' speeds.
  // How far that can even out the XCDs depends on the order of the work items: with small groups of
  // KV heads an XCD fetches few query rows but shares a KV head with few other XCDs; with one group
  // of all KV heads every XCD fetches every query row and all of them can be balanced against each
  // other.  Every group size (a power of two that divides the KV heads, or all of them) is tried, with
  // the XCDs in their own order and dealt to the groups by speed (deal_xcd_runs).
  double best = 0.0;
  int best_group = 0;
  for (int g = 1; g <= n_kv_heads; g = (2 * g <= n_kv_heads || g == n_kv_heads) ? 2 * g : n_kv_heads) {
    if (n_kv_heads % g) continue;
    const unsigned dealt = deal_xcd_runs(xcd_speed, tiles, n_kv_heads, n_splits, g);
    for (int k = 0; k < (dealt == kIdentityXcdRuns ? 1 : 2); ++k) {
      const unsigned runs = k ? dealt : kIdentityXcdRuns;
      uint32_t trial[kMaxCutHeads][33];
      const double t = try_kv_group(xcd_speed, tiles, n_kv_heads, n_splits, g, runs, std::max(1, max_nt), n_cu,
                                    q_bytes_per_kv_head, trial);
      if (!best_group || t < best - 1e-9) {
        best = t;
        best_group = g;
        *xcd_runs = runs;
        memcpy(cuts, trial, sizeof(trial));
      }
    }
  }
  *kv_group = best_group;
  *use = 1;
  return BA_OK;
}

int64_t build_final_meta(const int32_t *cu_q, const int32_t *cu_ctx, int n0, int n, int G, FinalMeta *meta) {
  memset(meta, 0, sizeof(*meta));
  meta->n = n;
  int64_t tiles = 0;
  for (int i = 0; i < n; ++i) {
    meta->cu_q[i] = cu_q[n0 + i];
    meta->cu_ctx[i] = cu_ctx[n0 + i];
    meta->tile_start[i] = (int32_t)tiles;
    tiles += ((int64_t)(cu_q[n0 + i + 1] - cu_q[n0 + i]) * G + kTileRows - 1) / kTileRows;
  }
  meta->cu_q[n] = cu_q[n0 + n];
  meta->cu_ctx[n] = cu_ctx[n0 + n];
  meta->tile_start[n] = (int32_t)tiles;
  return tiles;
}

int32_t plan_final_blocks(const ba_heads *h, int32_t n_prompts, const int32_t *cu_q, const int32_t *cu_blk,
                          const int32_t *blk_len, bool have_rot_out, int32_t gather_below, int n_cu,
                          BlocksPlan *plan) {
  if (gather_below < 0 && gather_below != BA_GATHER_DEFAULT)
    return fail(BA_ERR_INVALID_ARG, "gather_below %d: a token count, 0 or BA_GATHER_DEFAULT", gather_below);
  if (gather_below == BA_GATHER_DEFAULT) gather_below = 256;
  if (n_prompts < 0 || (n_prompts > 0 && (!cu_q || !cu_blk)))
    return fail(BA_ERR_INVALID_ARG, "cu_q / cu_blk: null or negative prompt count");
  BlocksPlan pl;
  if (n_prompts > 0 && (cu_q[0] != 0 || cu_blk[0] != 0)) return fail(BA_ERR_INVALID_ARG, "cu_q[0] and cu_blk[0] must be 0");
  const int G = h->n_q_heads / h->n_kv_heads;
  int64_t max_nb = 0;  // most non-empty blocks in one prompt
  for (int n = 0; n < n_prompts; ++n) {
    const int64_t lq = (int64_t)cu_q[n + 1] - cu_q[n];
    if (lq < 1) return fail(BA_ERR_INVALID_ARG, "prompt %d: the final block needs at least one token", n);
    if (cu_blk[n + 1] < cu_blk[n]) return fail(BA_ERR_INVALID_ARG, "prompt %d: cu_blk decreases", n);
    if (cu_blk[n + 1] > cu_blk[n] && !blk_len) return fail(BA_ERR_INVALID_ARG, "blk_len is null");
    if (lq * G > 0x3fffffff) return fail(BA_ERR_INVALID_ARG, "prompt %d: too many packed rows", n);
    int64_t tiles = (lq + kTileKeys - 1) / kTileKeys, ctx = 0, nb = 0;
    for (int b = cu_blk[n]; b < cu_blk[n + 1]; ++b) {
      if (blk_len[b] < 0) return fail(BA_ERR_INVALID_ARG, "block %d: negative length", b);
      if (blk_len[b] == 0) continue;
      tiles += (blk_len[b] + kTileKeys - 1) / kTileKeys;
      ctx += blk_len[b];
      ++nb;
    }
    if (ctx > 0x3fffffff || tiles > 0x1ffffff) return fail(BA_ERR_INVALID_ARG, "prompt %d: context too long", n);
    max_nb = std::max(max_nb, nb);
    pl.n_blocks += nb;
    pl.total_tiles += (lq * G + kTileRows - 1) / kTileRows;
    pl.max_nt = std::max(pl.max_nt, (int)tiles);
  }
  pl.lq_total = n_prompts > 0 ? cu_q[n_prompts] : 0;
  // The kernel that reads the block table pays a fixed price per block (it turns its queries at
  // every block boundary), a gathered copy a price per token: short blocks are gathered.
  int64_t ctx_total = 0;
  pl.cu_ctx.assign(n_prompts + 1, 0);
  for (int n = 0; n < n_prompts; ++n) {
    for (int b = cu_blk[n]; b < cu_blk[n + 1]; ++b) ctx_total += blk_len[b];
    if (ctx_total > 0x3fffffff) return fail(BA_ERR_INVALID_ARG, "context too long");
    pl.cu_ctx[n + 1] = (int32_t)ctx_total;
  }
  if (pl.n_blocks > 0 && ctx_total < (int64_t)gather_below * pl.n_blocks) {
    FinalPlan fp;
    int32_t rc = plan_final(h, n_prompts, cu_q, pl.cu_ctx.data(), BA_ROPE_APPLY, have_rot_out, n_cu, &fp);
    if (rc) return rc;
    pl.gather = true;
    pl.gather_kv_bytes = (size_t)ctx_total * h->n_kv_heads * h->head_dim * 2;
    pl.gather_final_bytes = fp.total();
    *plan = pl;
    return BA_OK;
  }
  if (max_nb > kBlkMaxBlocks)
    return fail(BA_ERR_UNSUPPORTED, "%lld cached blocks in one prompt, at most %d when the kernel reads the block table",
                (long long)max_nb, kBlkMaxBlocks);
  pl.n_splits = choose_splits(pl.total_tiles * h->n_kv_heads, pl.max_nt, n_cu);
  if (!have_rot_out) pl.kf_bytes = (size_t)pl.lq_total * h->n_kv_heads * h->head_dim * 2;
  pl.q_bytes = (size_t)pl.lq_total * h->n_q_heads * h->head_dim * 2;
  pl.rot_bytes = (size_t)pl.n_blocks * h->head_dim * 4;  // D/2 (cos, sin) pairs per block
  if (pl.n_splits > 1) {
    const size_t rows = partial_rows(pl.total_tiles, h->n_kv_heads);
    pl.part_o_bytes = (size_t)pl.n_splits * rows * h->head_dim * 2;
    pl.part_ml_bytes = (size_t)pl.n_splits * rows * 2 * 4;
    pl.part_idx_bytes = rows * 4;
  }
  *plan = pl;
  return BA_OK;
}

// Blocks up to kShortMaxLen tokens take the schedule with small workgroups, several to a compute
// unit; longer ones the main core.  (The short-block kernel assumes at most 8 tokens per 32 packed
// rows, and addresses the rows of a block with 32-bit element offsets.)
int64_t encode_short_max(int G, int64_t widest_stride) {
  return (G >= 4 && ((int64_t)kShortMaxLen + 1) * widest_stride < 0x40000000) ? kShortMaxLen : -1;
}

int32_t build_encode_metas(const int32_t *block_offsets, int b0, int n, int G, int64_t short_max, EncodeMeta meta[2],
                           int64_t tiles[2]) {
  tiles[0] = tiles[1] = 0;
  memset(meta, 0, 2 * sizeof(EncodeMeta));
  for (int i = 0; i < n; ++i) {
    const int64_t len = (int64_t)block_offsets[b0 + i + 1] - block_offsets[b0 + i];
    if (len * G > 0x3fffffff) return fail(BA_ERR_INVALID_ARG, "block %d: too many packed rows", b0 + i);
    const int which = len <= short_max ? 1 : 0;
    for (int m = 0; m < 2; ++m) {
      meta[m].offs[i] = block_offsets[b0 + i];
      meta[m].tile_start[i] = (int32_t)tiles[m];
    }
    const int tile_rows = which ? kShortTileRows : kTileRows;
    tiles[which] += (len * G + tile_rows - 1) / tile_rows;
    if (tiles[which] > 0x3fffffff) return fail(BA_ERR_INVALID_ARG, "too many row tiles in one call");
  }
  for (int m = 0; m < 2; ++m) {
    meta[m].n = n;
    meta[m].offs[n] = block_offsets[b0 + n];
    meta[m].tile_start[n] = (int32_t)tiles[m];
    for (int i = n + 1; i <= kEncMaxBlocks; ++i) meta[m].tile_start[i] = 0x7fffffff;
  }
  return BA_OK;
}

std::vector<PromptBlock> list_prompt_blocks(int32_t n_prompts, const int32_t *cu_blk, const int32_t *block_offsets) {
  std::vector<PromptBlock> blks;
  for (int n = 0; n < n_prompts; ++n) {
    const int last = cu_blk[n + 1] - 1;
    const int32_t fs = block_offsets[last], fl = block_offsets[last + 1] - fs;
    for (int b = cu_blk[n]; b <= last; ++b) {
      const int32_t len = block_offsets[b + 1] - block_offsets[b];
      if (len == 0) continue;
      // first key a block sees: its own first token, or for a prompt's last block the prompt's
      blks.push_back({block_offsets[b], len, b == last ? block_offsets[cu_blk[n]] : block_offsets[b], fs,
                      b == last ? 0 : fl, n});
    }
  }
  return blks;
}

void sort_by_key_range(std::vector<PromptBlock> *blks) {
  // (a prompt's last block walks the whole prompt, and a launch should not end on a few of those)
  std::stable_sort(blks->begin(), blks->end(), [](const PromptBlock &a, const PromptBlock &b) {
    return (int64_t)a.start + a.len - a.kstart > (int64_t)b.start + b.len - b.kstart;
  });
}

int64_t build_prompt_meta(const std::vector<PromptBlock> &blks, size_t b0, int n, int G, PromptMeta *meta) {
  memset(meta, 0, sizeof(*meta));
  meta->n = n;
  int64_t tiles = 0;
  for (int i = 0; i < n; ++i) {
    meta->start[i] = blks[b0 + i].start;
    meta->len[i] = blks[b0 + i].len;
    meta->kstart[i] = blks[b0 + i].kstart;
    meta->tile_start[i] = (int32_t)tiles;
    tiles += ((int64_t)blks[b0 + i].len * G + kShortTileRows - 1) / kShortTileRows;
    if (tiles > 0x3fffffff) return -1;
  }
  meta->tile_start[n] = (int32_t)tiles;
  for (int i = n + 1; i <= kEncMaxBlocks; ++i) meta->tile_start[i] = 0x7fffffff;
  return tiles;
}

namespace {

// largest i < n with tile_start[i] <= tile: what the kernels look up
int segment_of(const int32_t *tile_start, int n, int tile) {
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tile_start[mid] <= tile) lo = mid; else hi = mid;
  }
  return lo;
}

struct ItemSink {
  ba_work_item *out;
  int64_t max, n = 0;
  void put(const ba_work_item &w) {
    if (out && n < max) out[n] = w;
    ++n;
  }
};

}  // namespace
}  // namespace ba

extern "C" {

const char *ba_last_error(void) { return ba::last_error(); }

int64_t ba_schedule_final_block(const ba_heads *heads, int32_t n_prompts, const int32_t *cu_q, const int32_t *cu_ctx,
                                int32_t n_compute_units, ba_work_item *items, int64_t max_items) {
  int32_t rc;
  if ((rc = ba::check_heads(heads, true))) return rc;
  if (n_compute_units < 1) return ba::fail(BA_ERR_INVALID_ARG, "n_compute_units must be positive");
  ba::FinalPlan pl;
  if ((rc = ba::plan_final(heads, n_prompts, cu_q, cu_ctx, BA_ROPE_APPLY, false, n_compute_units, &pl))) return rc;
  const int G = heads->n_q_heads / heads->n_kv_heads;
  ba::ItemSink sink{items, items ? max_items : 0};
  int launch = 0;
  for (int n0 = 0; n0 < n_prompts; n0 += ba::kFinMaxPrompts, ++launch) {
    const int n = std::min(ba::kFinMaxPrompts, n_prompts - n0);
    ba::FinalMeta meta;
    const int64_t tiles = ba::build_final_meta(cu_q, cu_ctx, n0, n, G, &meta);
    uint32_t cuts[ba::kMaxCutHeads][33];
    int32_t use_cuts = 0;
    int32_t kv_group = 0;
    uint32_t xcd_runs = ba::kIdentityXcdRuns;
    if ((rc = ba::plan_split_cuts(heads->xcd_speed, tiles, heads->n_kv_heads, pl.n_splits, pl.max_nt, n_compute_units,
                                  ba::final_q_bytes_per_kv_head(heads, pl.lq_total), cuts, &use_cuts, &kv_group, &xcd_runs)))
      return rc;
    // the kernel's own walk: every (split, row tile) of the launch; the same at every KV head unless
    // the splits are sized by XCD speed, when every KV head has shares of its own
    const ba::ItemOrder order = {(int)tiles, heads->n_kv_heads, pl.n_splits, kv_group};
    const int64_t n_wg = tiles * heads->n_kv_heads * pl.n_splits;
    for (int kvh = use_cuts ? 0 : -1; kvh < (use_cuts ? heads->n_kv_heads : 0); ++kvh)
    for (int split = 0; split < pl.n_splits; ++split)
      for (int64_t tile = 0; tile < tiles; ++tile) {
        const int i = ba::segment_of(meta.tile_start, meta.n, (int)tile);
        const int lq = meta.cu_q[i + 1] - meta.cu_q[i], tctx = meta.cu_ctx[i + 1] - meta.cu_ctx[i];
        const int jt = (int)tile - meta.tile_start[i];
        const int n_rows = lq * G, row0 = jt * ba::kTileRows;
        const int last_row = std::min(n_rows, row0 + ba::kTileRows) - 1;
        const int n_ctx_tiles = (tctx + ba::kTileKeys - 1) / ba::kTileKeys;
        const int n_causal = ba::causal_key_tiles(last_row / G, ba::kTileKeys);
        const ba::TileRange tr = ba::split_tile_range(n_ctx_tiles, n_causal, pl.n_splits, split, use_cuts ? cuts[kvh] : nullptr);
        ba_work_item w;
        memset(&w, 0, sizeof(w));
        w.launch = launch;
        w.problem = n0 + i;
        w.first_token = meta.cu_q[i];
        w.tile_rows = ba::kTileRows;
        w.tile_keys = ba::kTileKeys;
        w.row_begin = row0;
        w.row_end = last_row + 1;
        w.split = split;
        w.n_splits = pl.n_splits;
        w.kv_head = kvh;
        w.xcd = kvh >= 0 && n_wg <= 0x7fffffff
                    ? ba::xcd_of_work_item(ba::item_id((int)tile, kvh, split, order), (unsigned)n_wg, xcd_runs) : -1;
        w.ctx_begin = std::min(tctx, std::min(tr.begin, n_ctx_tiles) * ba::kTileKeys);
        w.ctx_end = std::min(tctx, std::min(tr.end, n_ctx_tiles) * ba::kTileKeys);
        w.self_begin = std::min(lq, std::max(0, tr.begin - n_ctx_tiles) * ba::kTileKeys);
        w.self_end = std::min(lq, std::max(0, tr.end - n_ctx_tiles) * ba::kTileKeys);
        sink.put(w);
      }
  }
  return sink.n;
}

int64_t ba_schedule_encode_blocks(const ba_heads *heads, int32_t n_blocks, const int32_t *block_offsets,
                                  ba_work_item *items, int64_t max_items) {
  int32_t rc;
  if ((rc = ba::check_heads(heads, true))) return rc;
  if ((rc = ba::check_offsets(n_blocks, block_offsets))) return rc;
  const int G = heads->n_q_heads / heads->n_kv_heads;
  const int64_t short_max = ba::encode_short_max(G, (int64_t)heads->n_q_heads * heads->head_dim);
  ba::ItemSink sink{items, items ? max_items : 0};
  int launch = 0;
  for (int b0 = 0; b0 < n_blocks; b0 += ba::kEncMaxBlocks) {
    const int n = std::min(ba::kEncMaxBlocks, n_blocks - b0);
    ba::EncodeMeta meta[2];
    int64_t tiles[2];
    if ((rc = ba::build_encode_metas(block_offsets, b0, n, G, short_max, meta, tiles))) return rc;
    for (int m = 1; m >= 0; --m) {
      if (tiles[m] == 0) continue;
      const int tile_rows = m ? ba::kShortTileRows : ba::kTileRows, tile_keys = m ? 32 : ba::kTileKeys;
      for (int64_t tile = 0; tile < tiles[m]; ++tile) {
        const int i = ba::segment_of(meta[m].tile_start, meta[m].n, (int)tile);
        const int lq = meta[m].offs[i + 1] - meta[m].offs[i];
        const int jt = (int)tile - meta[m].tile_start[i];
        const int n_rows = lq * G, row0 = jt * tile_rows;
        const int last_row = std::min(n_rows, row0 + tile_rows) - 1;
        ba_work_item w;
        memset(&w, 0, sizeof(w));
        w.kv_head = w.xcd = -1;
        w.launch = launch;
        w.problem = b0 + i;
        w.first_token = meta[m].offs[i];
        w.tile_rows = tile_rows;
        w.tile_keys = tile_keys;
        w.row_begin = row0;
        w.row_end = last_row + 1;
        w.n_splits = 1;
        w.self_end = std::min(lq, ba::causal_key_tiles(last_row / G, tile_keys) * tile_keys);
        sink.put(w);
      }
      ++launch;
    }
  }
  return sink.n;
}

int64_t ba_schedule_prompts(const ba_heads *heads, int32_t n_prompts, const int32_t *cu_blk,
                            const int32_t *block_offsets, ba_work_item *items, int64_t max_items) {
  int32_t rc;
  if ((rc = ba::check_heads(heads, true))) return rc;
  if ((rc = ba::check_prompt_blocks(n_prompts, cu_blk, block_offsets))) return rc;
  const int G = heads->n_q_heads / heads->n_kv_heads;
  std::vector<ba::PromptBlock> blks = ba::list_prompt_blocks(n_prompts, cu_blk, block_offsets);
  ba::sort_by_key_range(&blks);
  ba::ItemSink sink{items, items ? max_items : 0};
  int launch = 0;
  for (size_t b0 = 0; b0 < blks.size(); b0 += ba::kEncMaxBlocks, ++launch) {
    const int n = (int)std::min<size_t>(ba::kEncMaxBlocks, blks.size() - b0);
    ba::PromptMeta meta;
    const int64_t tiles = ba::build_prompt_meta(blks, b0, n, G, &meta);
    if (tiles < 0) return ba::fail(BA_ERR_INVALID_ARG, "too many row tiles in one call");
    for (int64_t tile = 0; tile < tiles; ++tile) {
      const int i = ba::segment_of(meta.tile_start, meta.n, (int)tile);
      const int lq = meta.len[i], dq = meta.start[i] - meta.kstart[i];  // dq: earlier tokens of the prompt it sees
      const int jt = (int)tile - meta.tile_start[i];
      const int n_rows = lq * G, row0 = jt * ba::kShortTileRows;
      const int last_row = std::min(n_rows, row0 + ba::kShortTileRows) - 1;
      // keys counted from the first visible one: tiles up to the one that holds the last row's own token
      const int keys_walked = ((dq + last_row / G) / 32 + 1) * 32;
      ba_work_item w;
      memset(&w, 0, sizeof(w));
      w.kv_head = w.xcd = -1;
      w.launch = launch;
      w.problem = blks[b0 + i].prompt;
      w.first_token = meta.start[i];
      w.tile_rows = ba::kShortTileRows;
      w.tile_keys = 32;
      w.row_begin = row0;
      w.row_end = last_row + 1;
      w.n_splits = 1;
      w.ctx_begin = 0;
      w.ctx_end = std::min(dq, keys_walked);
      w.self_end = std::min(lq, std::max(0, keys_walked - dq));
      sink.put(w);
    }
  }
  return sink.n;
}

}  // extern "C"
