// Host-side planning of the Block-attention calls: argument checks on the host arrays, the number of
// KV splits, workspace layouts, and the tables of row tiles that travel to the kernels.  Nothing here
// touches a device: every function runs on a machine without a GPU, which is how it is tested
// (the work items of a plan must cover exactly the visible pairs of the block mask).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/ba.h"
#include "ba_internal.h"
#include "ba_schedule.h"

namespace ba {

// Status + thread-local message (what ba_last_error() returns).
int32_t fail(int32_t status, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
const char *last_error();

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Split partials are kept per row tile (whole tiles, also where a problem's last tile is ragged):
// packed rows they cover, over all KV heads.
inline size_t partial_rows(int64_t total_tiles, int n_kv_heads) { return (size_t)total_tiles * n_kv_heads * kTileRows; }

int32_t check_heads(const ba_heads *h, bool attention);
// block_offsets of n_blocks blocks: starts at 0, never decreases
int32_t check_offsets(int32_t n_blocks, const int32_t *offs);
// cu_blk of a whole-prompt call (cu_blk[0] = 0, at least one block per prompt) and the offsets behind it
int32_t check_prompt_blocks(int32_t n_prompts, const int32_t *cu_blk, const int32_t *block_offsets);

// Number of KV splits of a final-block launch of base_wgs workgroups (row tiles x KV heads) whose
// longest walk has max_tiles key tiles, on a device of n_cu compute units.
int choose_splits(int64_t base_wgs, int max_tiles, int n_cu);

struct FinalPlan {
  int64_t lq_total = 0;
  int64_t total_tiles = 0;  // row tiles over all prompts
  int max_nt = 0;           // longest walk, key tiles
  int n_splits = 1;
  size_t kf_bytes = 0, q_bytes = 0, part_o_bytes = 0, part_ml_bytes = 0, part_idx_bytes = 0;
  size_t total() const {
    return align256(kf_bytes) + align256(q_bytes) + align256(part_o_bytes) + align256(part_ml_bytes) +
           align256(part_idx_bytes);
  }
};
int32_t plan_final(const ba_heads *h, int32_t n_prompts, const int32_t *cu_q, const int32_t *cu_ctx,
                   int32_t rope_mode, bool have_rot_out, int n_cu, FinalPlan *plan);
// Order of the work items and shares of the KV splits of one final-block launch (tiles row tiles x
// n_kv_heads KV heads x n_splits splits, one workgroup each; the longest walk is max_nt key tiles) on
// a device of n_cu compute units.  xcd_speed: eight positive numbers or null.  With speeds the
// splits of every KV head are sized by the speed of the XCDs that run them: cuts[h][s] = where split s
// of KV head h begins, 1 / 65536 units (see split_tile_range), and *kv_group (see ItemOrder) is the
// group size under which the launch is expected to end soonest.  *use = 0 when the splits stay equal
// (no speeds, one split, too many KV heads): then *kv_group is the default.  *xcd_runs: which run of
// work items each XCD takes (work_item_of_workgroup; the identity unless a deal by speed is expected to
// end sooner).  BA_ERR_INVALID_ARG on bad speeds.  q_bytes_per_kv_head: the query rows a workgroup's
// XCD fetches per KV head it hosts.
int32_t plan_split_cuts(const float *xcd_speed, int64_t tiles, int n_kv_heads, int n_splits, int max_nt, int n_cu,
                        double q_bytes_per_kv_head, uint32_t cuts[kMaxCutHeads][33], int32_t *use, int32_t *kv_group,
                        uint32_t *xcd_runs);
inline double final_q_bytes_per_kv_head(const ba_heads *h, int64_t lq_total) {
  return (double)lq_total * (h->n_q_heads / h->n_kv_heads) * h->head_dim * 2.0;
}
// The table of one final-block launch: prompts [n0, n0 + n).  Returns its row tiles.
int64_t build_final_meta(const int32_t *cu_q, const int32_t *cu_ctx, int n0, int n, int G, FinalMeta *meta);

struct BlocksPlan {
  int64_t lq_total = 0;
  int64_t total_tiles = 0;
  int64_t n_blocks = 0;  // non-empty blocks over all prompts
  int max_nt = 0;
  int n_splits = 1;
  size_t kf_bytes = 0, q_bytes = 0, rot_bytes = 0, part_o_bytes = 0, part_ml_bytes = 0, part_idx_bytes = 0;
  // Small blocks: the context is first gathered (K re-encoded, V copied) into the workspace and the
  // call continues as ba_final_block_attention.
  bool gather = false;
  std::vector<int32_t> cu_ctx;    // per prompt, gathered route only
  size_t gather_kv_bytes = 0;     // one of the two gathered tensors
  size_t gather_final_bytes = 0;  // workspace of the final-block step behind them
  size_t total() const {
    if (gather) return 2 * align256(gather_kv_bytes) + gather_final_bytes;
    return align256(kf_bytes) + align256(q_bytes) + align256(rot_bytes) + align256(part_o_bytes) +
           align256(part_ml_bytes) + align256(part_idx_bytes);
  }
};
// gather_below: mean length (tokens) of a call's cached blocks below which the call gathers
// (BA_GATHER_DEFAULT: 256; 0: never).
int32_t plan_final_blocks(const ba_heads *h, int32_t n_prompts, const int32_t *cu_q, const int32_t *cu_blk,
                          const int32_t *blk_len, bool have_rot_out, int32_t gather_below, int n_cu,
                          BlocksPlan *plan);

// Per-block encoding, blocks [b0, b0 + n): one table per schedule ([0] main core, [1] short blocks;
// a block has row tiles in the table of its own schedule only).  short_max: longest block (tokens)
// the short-block schedule takes, -1 for none.
int32_t build_encode_metas(const int32_t *block_offsets, int b0, int n, int G, int64_t short_max, EncodeMeta meta[2],
                           int64_t tiles[2]);
// Longest block the short-block schedule takes at these strides (elements) and this group size.
int64_t encode_short_max(int G, int64_t widest_stride);

// Whole prompts (Section 2.4): non-empty blocks with the first key they see and (for passages) their
// prompt's last block.
struct PromptBlock {
  int32_t start, len, kstart, fin_start, fin_len, prompt;
};
std::vector<PromptBlock> list_prompt_blocks(int32_t n_prompts, const int32_t *cu_blk, const int32_t *block_offsets);
// ... in the order the forward and dq kernels take them (longest key range first)
void sort_by_key_range(std::vector<PromptBlock> *blks);
// the table of one launch: blocks [b0, b0 + n) of the list.  Returns its row tiles, -1 if too many.
int64_t build_prompt_meta(const std::vector<PromptBlock> &blks, size_t b0, int n, int G, PromptMeta *meta);

}  // namespace ba
