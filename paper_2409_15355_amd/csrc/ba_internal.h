// Internal interface between the C boundary (ba_api.hip) and the gfx950 kernels.
// Small per-call metadata travels BY VALUE in the kernel-argument segment, so no call
// ever copies host memory to the device or needs device-side scratch for schedules;
// long block lists are cut into several launches by the host code.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ba_schedule.h"

namespace ba {

constexpr int kMaxFreq = 64;  // head_dim / 2 <= 64

// theta_j / (2*pi) as an unsigned Q0.64 fraction of a turn.  position * turns[j]
// (mod 2^64) is then the exact phase of the RoPE angle position * theta_j (Eq. 1).
struct RopeTable {
  uint64_t turns[kMaxFreq];
};

// ---------------------------------------------------------------- re-encode ----------
// Two capacities (the table travels by value in the kernel arguments): retrieval-sized block lists,
// and the long lists of small blocks that a gathered context is made of.
constexpr int kReencMaxBlocks = 96, kReencMaxBlocksLarge = 1024;

template <int NB>
struct ReencBlocksT {
  static constexpr int kBlocks = NB;
  int32_t n;
  int32_t src_off[NB];
  int32_t dst_off[NB];
  int32_t len[NB];
  int32_t pos_old[NB];
  int32_t pos_new[NB];
};
using ReencBlocks = ReencBlocksT<kReencMaxBlocks>;
using ReencBlocksLarge = ReencBlocksT<kReencMaxBlocksLarge>;

struct ReencParams {
  const void *src;
  void *dst;
  int64_t src_st, src_sh, dst_st, dst_sh;  // token / head strides, elements
  int64_t src_sl, dst_sl;                  // layer strides, elements
  int32_t n_layers, n_kv_heads, head_dim;
  int32_t dtype, layout, mode;
  int32_t max_len;  // longest block in this launch
  int32_t heads_per_thread, n_head_groups;  // how the KV heads are split over workgroups
  int32_t copy_from_layer;  // layers from this one on are copied as they are (a gathered V rides along as a layer)
};

hipError_t launch_reencode(const ReencParams &p, const ReencBlocks &blocks, const RopeTable &rt,
                           hipStream_t stream);
hipError_t launch_reencode(const ReencParams &p, const ReencBlocksLarge &blocks, const RopeTable &rt,
                           hipStream_t stream);

// Final block over a block table: prompts and cached blocks per launch.  Two capacities, because
// the tables travel by value in the kernel arguments and many large argument blocks in flight
// throttle the launch queue: the small one covers retrieval-sized prompts.
constexpr int kBlkMaxPrompts = 64, kBlkMaxBlocks = 1024;
constexpr int kBlkSmallPrompts = 16, kBlkSmallBlocks = 64;

// ---------------------------------------------------------------- RoPE pre-pass ------
// Fresh (un-rotated) Q and K rows of a run of consecutive segments: segment s covers tokens
// [start[s], start[s+1]) and its first token has position pos0[s].
constexpr int kRopeMaxSegs = 320;

// (two capacities: the table travels by value in the kernel arguments, and a final-block call of a
// few prompts should not carry 2.5 KB of it through every launch)
template <int N>
struct RopeSegsT {
  static constexpr int kSegs = N;
  int32_t n;
  int32_t start[N + 1];
  int32_t pos0[N];
};
using RopeSegs = RopeSegsT<kRopeMaxSegs>;
constexpr int kRopeSmallSegs = 8;
using RopeSegsSmall = RopeSegsT<kRopeSmallSegs>;

struct RopePrepassParams {
  const uint16_t *q_src;
  uint16_t *q_dst;
  int64_t q_st, q_sh, qd_st, qd_sh;  // token / head strides, elements
  const uint16_t *k_src;
  uint16_t *k_dst;
  int64_t k_st, k_sh, kd_st, kd_sh;
  float q_scale;  // Q is multiplied by this before its one rounding
  int32_t n_q_heads, n_kv_heads, head_dim, layout;
  int32_t heads_per_thread;
  int32_t do_q, do_k;
  float *rot_dst;    // [n_rot][D/2][2]: (cos, sin) of rot_angle[b] * theta_j, or null
  int32_t n_rot;
  float *q_table;    // do_q == 2: instead of rotating Q rows, write q_scale * (cos, sin) per token: [tokens][D/2][2];
                     // do_q == 3: both the rotated rows and the table;
                     // do_q == 4: the table only, by position: row r = q_scale * (cos, sin) of position r,
                     //            r < table_rows (for calls all of whose segments start at position 0)
  int32_t table_rows;
};

// positions (in tokens) by which the rows of the rotation table turn
template <int NB>
struct RopeRotsT {
  int32_t angle[NB];
};
using RopeRots = RopeRotsT<kBlkMaxBlocks>;
using RopeRotsSmall = RopeRotsT<kBlkSmallBlocks>;

// rots / rots_small: at most one non-null, and only with p.rot_dst
hipError_t launch_rope_prepass(const RopePrepassParams &p, const RopeSegs &segs, const RopeRots *rots,
                               const RopeRotsSmall *rots_small, const RopeTable &rt, hipStream_t stream);
hipError_t launch_rope_prepass(const RopePrepassParams &p, const RopeSegsSmall &segs, const RopeRots *rots,
                               const RopeRotsSmall *rots_small, const RopeTable &rt, hipStream_t stream);

// ---------------------------------------------------------------- shared by the files of the boundary ----
int32_t device_fail(hipError_t e, const char *what);  // BA_ERR_DEVICE with the runtime's text
int num_cus();                                        // compute units of the current device
unsigned long long *&probe_clock();                   // this thread's AttnParams::wg_clock for the next final-block launches

// ---------------------------------------------------------------- attention ----------

constexpr int kProbeRecord = 16;
constexpr int kTileRows = 256;  // packed (token, head-in-group) query rows per workgroup
constexpr int kTileKeys = 64;   // keys per K/V tile
constexpr int kShortTileRows = 128;  // packed query rows per workgroup of the short-block schedule
// Per-block encoding sends blocks up to this length through the short-block schedule (measured
// crossover: beyond about 6,000 to 8,000 tokens the deep pipeline of the main core wins).
constexpr int kShortMaxLen = 6144;

struct AttnParams {
  const uint16_t *q;
  int64_t q_st, q_sh;
  const uint16_t *kc;  // context keys / values (final block only; used as given)
  int64_t kc_st, kc_sh;
  const uint16_t *vc;
  int64_t vc_st, vc_sh;
  const uint16_t *kf;  // causal-segment keys / values (already rotated)
  int64_t kf_st, kf_sh;
  const uint16_t *vf;
  int64_t vf_st, vf_sh;
  uint16_t *o;
  int64_t o_st, o_sh;
  // Split partials, per "unit" = the 32 packed rows one wave owns: unit = ((tile_base + row tile) *
  // n_kv_heads + KV head) * 8 + wave.  A split's normalised output stays in the layout the MFMA
  // accumulators have (no transposition on the way out; every wave instruction stores 1 KB of
  // consecutive memory); the merge kernel reads that layout back and writes the rows where they belong.
  uint16_t *part_o;   // [n_splits][part_units][D / 16][64 lanes][8] fp16
  float *part_ml;     // [n_splits][part_units][32][2]  (reference in log2 units, sum of exponentials)
  int32_t *part_idx;  // [part_units][32]  output row (token * n_q_heads + head) of each packed row, -1: none
  int64_t part_units;
  int32_t tile_base;  // row tiles of the call's earlier launches
  int32_t n_q_heads, n_kv_heads, group, head_dim;
  FastDiv group_div;  // division by `group`
  float scale_log2e;  // softmax scale * log2(e)
  int32_t q_ready;    // q is already rotated and multiplied by scale_log2e (the RoPE pre-pass ran)
  int32_t q_rows_fit32;  // main core, filled at the launch: 32 tokens and a group of heads of q span less than 2^32 bytes
  const float *q_table;  // else, if non-null: [tokens][D/2][2] = scale_log2e * (cos, sin) of each
                         // token's position times theta_j; the kernel rotates q with it
  int32_t q_table_by_pos;  // ... or, if set, [positions][D/2][2]: a row per position inside the block (per-block
                           // encoding, where every block starts at position 0 and the blocks share one table)
  int32_t rope_layout;
  const float *blk_rot;  // block table only: [blocks][D/2][2] (cos, sin) of minus each block's shift
  int32_t n_splits;
  int32_t use_cuts;            // split_cut holds unequal shares (see split_tile_range)
  uint32_t split_cut[kMaxCutHeads][33];  // per KV head: cumulative shares of its splits, 1 / 65536 units
  unsigned long long *wg_clock;  // probe only, else null: kProbeRecord numbers per workgroup:
                                 // [0] XCC id, [1] shader cycles and [2] 100 MHz ticks at entry, [4] and [5] the same
                                 // behind the walk, ticks [3] first tile copies issued, [6] first tiles and query
                                 // fragments landed, [7] loop entered, [8] partials' stores issued, [9] complete
  int32_t total_tiles;  // row tiles over all problems of this launch
  FastDiv tiles_div;    // division by total_tiles
  int32_t kv_group;     // main core, filled at the launch: KV heads per group in the order of the work items
  uint32_t xcd_runs;    // main core: which run of work items each XCD takes (work_item_of_workgroup); 0 = in order
  ItemDivs item_divs;   // ... and the divisors of item_coords
  SplitDivs split_divs; // divisions by n_splits and 2 n_splits (main core; filled at the launch)
  float *lse;           // short-block schedule: [tokens][n_q_heads] log-sum-exp of the scaled scores, or null
};

constexpr int kEncMaxBlocks = 320;
struct EncodeMeta {
  int32_t n;
  int32_t offs[kEncMaxBlocks + 1];        // token offsets of the blocks
  int32_t tile_start[kEncMaxBlocks + 1];  // first row tile of each block; [n] = all tiles, INT_MAX beyond
};

// Whole prompts (Section 2.4): blocks in any order (the host lists the ones with the longest key
// ranges first), each with its first token, its length and the first key it sees.
struct PromptMeta {
  int32_t n;
  int32_t start[kEncMaxBlocks];
  int32_t len[kEncMaxBlocks];
  int32_t tile_start[kEncMaxBlocks + 1];  // in row tiles of kShortTileRows rows; INT_MAX beyond [n]
  int32_t kstart[kEncMaxBlocks];          // token offset of the first visible key
};

// ---------------------------------------------------------------- backward of whole prompts ----
struct BwdParams {
  const uint16_t *dout;  // gradient of the output, [T][n_q_heads][D] with these strides
  int64_t do_st, do_sh;
  const uint16_t *o;     // the forward output, [T][n_q_heads][D] with these strides
  int64_t o_st, o_sh;
  const float *lse;      // [T][n_q_heads]: the forward pass's log-sum-exps
  float2 *ld;            // [n_kv_heads][T][group]: (log-sum-exp / ln 2, delta) of query head kvh * group + g,
                         // written by the dq kernel, read by the dk/dv kernel
  int64_t T;
  uint16_t *dq, *dk, *dv;  // the gradients, with these strides
  int64_t dq_st, dq_sh, dk_st, dk_sh, dv_st, dv_sh;
  float scale;           // softmax scale
};

// Owners of keys: blocks in any order, and for a passage the last block of its prompt (whose rows
// see the passage's keys as well).
struct BwdKvMeta {
  int32_t n;
  int32_t start[kEncMaxBlocks];
  int32_t len[kEncMaxBlocks];
  int32_t tile_start[kEncMaxBlocks + 1];  // in key tiles of kShortTileRows keys
  int32_t fin_start[kEncMaxBlocks];
  int32_t fin_len[kEncMaxBlocks];          // 0: the block is its prompt's last
};

hipError_t launch_bwd_dq(const AttnParams &p, const PromptMeta &meta, const BwdParams &bp, hipStream_t stream);
hipError_t launch_bwd_dkv(const AttnParams &p, const BwdKvMeta &meta, const BwdParams &bp, hipStream_t stream);

constexpr int kFinMaxPrompts = 64;
struct FinalMeta {
  int32_t n;
  int32_t cu_q[kFinMaxPrompts + 1];
  int32_t cu_ctx[kFinMaxPrompts + 1];
  int32_t tile_start[kFinMaxPrompts + 1];
};

// Final block over a table of cached blocks (each at the positions it was encoded at).
template <int NP, int NB>
struct FinalBlocksMetaT {
  static constexpr int kPrompts = NP, kBlocks = NB;
  int32_t n;
  int32_t rot_base;            // row of AttnParams::blk_rot that belongs to block 0 of this launch
  int32_t cu_q[NP + 1];
  int32_t cu_blk[NP + 1];      // blocks of prompt n: [cu_blk[n], cu_blk[n+1])
  int32_t ctx_tiles[NP];       // key tiles of prompt n's context
  int32_t tile_start[NP + 1];  // first row tile of each prompt
  int32_t blk_off[NB];         // first cache row of the block
  int32_t blk_len[NB];         // rows (>= 1)
  int32_t blk_tile0[NB];       // first key tile of the block inside its prompt
};
using FinalBlocksMeta = FinalBlocksMetaT<kBlkMaxPrompts, kBlkMaxBlocks>;
using FinalBlocksMetaSmall = FinalBlocksMetaT<kBlkSmallPrompts, kBlkSmallBlocks>;

// Rows of [tokens][heads][chunks * 16 bytes] tensors moved between a caller's tensor with `group`
// query heads per KV head and a packed one with `group_padded` (phantom heads are zero).
struct HeadPadParams {
  void *real;          // [tokens][n_kv_heads * group] rows, strides in elements of `elt` bytes
  int64_t real_st, real_sh;
  void *padded;        // [tokens][n_kv_heads * group_padded] rows
  int64_t padded_st, padded_sh;
  int64_t tokens;
  int32_t n_kv_heads, group, group_padded;
  int32_t chunks;      // 16-byte pieces per row
  int32_t elt;         // bytes per element (strides are in elements)
};
// to_padded: real -> padded (phantoms zeroed); else padded -> real (real heads only)
hipError_t launch_pad_heads(const HeadPadParams &p, bool to_padded, hipStream_t stream);
// the same for [tokens][heads] floats (real: packed [tokens][n_kv_heads * group])
hipError_t launch_pad_lse(float *real, float *padded, int64_t tokens, int n_kv_heads, int group, int group_padded,
                          bool to_padded, hipStream_t stream);

// MFMA rate diagnostic (diag.hip): n_wg workgroups of 8 waves, `iters` x 16 MFMAs each, with
// reads_per_two (0, 1, 2) LDS fragment reads per two MFMAs; per wave (shader cycles, 100 MHz ticks) into ws
size_t diag_mfma_workspace_bytes(int n_wg);
hipError_t launch_mfma_ceiling(int reads_per_two, int n_wg, int iters, void *ws, uint32_t seed, hipStream_t stream);

// n pseudo-random bf16 values (synthetic operands of the XCD speed probe)
hipError_t launch_fill_random_bf16(uint16_t *dst, int64_t n, uint32_t seed, hipStream_t stream);

hipError_t launch_attn_encode(const AttnParams &p, const EncodeMeta &meta, hipStream_t stream);
// the same for short blocks: meta.tile_start counts row tiles of kShortTileRows rows
hipError_t launch_attn_encode_short(const AttnParams &p, const EncodeMeta &meta, hipStream_t stream);
hipError_t launch_attn_prompt_short(const AttnParams &p, const PromptMeta &meta, hipStream_t stream);
hipError_t launch_attn_final_blocks(const AttnParams &p, const FinalBlocksMeta &meta, hipStream_t stream);
hipError_t launch_attn_final_blocks(const AttnParams &p, const FinalBlocksMetaSmall &meta, hipStream_t stream);
hipError_t launch_attn_final(const AttnParams &p, const FinalMeta &meta, hipStream_t stream);
// Merge the split-KV partials of all p.part_units units into the bf16 output.
hipError_t launch_combine(const AttnParams &p, hipStream_t stream);

}  // namespace ba
