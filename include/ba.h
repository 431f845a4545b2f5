/*
 * ba.h -- C boundary of the MI355X (gfx950) Block-attention prefill library.
 *
 * Block-attention (arXiv 2409.15355) splits a prompt into blocks: every block but
 * the last is encoded on its own (Section 2.1), its cached keys are rotated to the
 * block's place in the new prompt (Section 2.3, Eq. 1-3), and only the last block --
 * the user query -- attends to everything before it (Section 2.5).  The three entry
 * points below are those three steps.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * - Tensors are DEVICE memory described by `ba_tensor`: element pointer, token and head
 *   strides in ELEMENTS, innermost head_dim contiguous.  The default packed layout is
 *   [tokens][heads][head_dim] (stride_head = head_dim, stride_tok = heads * head_dim).
 *   Base pointers and both strides must be 16-byte aligned.
 * - Small metadata arrays (block offsets, per-block descriptors, cu_* arrays, q_to_kv,
 *   inv_freq) are HOST memory.  They are read and validated before the call returns
 *   and may be freed immediately afterwards.
 * - The caller owns all device memory, including the workspace; the library allocates
 *   nothing on the device and keeps no device state between calls.
 * - `stream` is a hipStream_t (NULL = the default stream).  All device work is
 *   enqueued on it; calls return without synchronising.
 * - Every call returns BA_OK or a negative status; nothing aborts or throws.
 *   `ba_last_error()` gives a thread-local description of the last failure.
 * - Outputs are fully overwritten for every row the call covers.
 * - Supported: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads; query head h
 *   uses KV head h / (n_q_heads / n_kv_heads) (a q_to_kv map is accepted only if it
 *   says exactly that).
 */
#ifndef BA_H_
#define BA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BA_OK 0
#define BA_ERR_INVALID_ARG (-1) /* null pointer, non-monotone offsets, bad head counts ... */
#define BA_ERR_UNSUPPORTED (-2) /* head_dim, dtype or head map outside what is built      */
#define BA_ERR_ALIGNMENT (-3)   /* pointer or stride not 16-byte aligned                   */
#define BA_ERR_WORKSPACE (-4)   /* workspace missing or too small                          */
#define BA_ERR_DEVICE (-5)      /* a HIP call failed; see ba_last_error()                  */

#define BA_DTYPE_BF16 0
#define BA_DTYPE_F32 1 /* ba_reencode_positions only */

#define BA_ROPE_INTERLEAVED 0 /* Eq. 1: dimension pairs (2j, 2j+1)                  */
#define BA_ROPE_HALF 1        /* pairs (j, j + head_dim/2), as Llama checkpoints store */

#define BA_ROPE_NONE 0  /* q and k arrive already rotated                               */
#define BA_ROPE_APPLY 1 /* rotate inside: local positions in ba_encode_blocks (first token
                           of a block at 0, Section 2.3), absolute positions in
                           ba_final_block_attention                                    */

#define BA_REENC_SHIFT 0    /* cache holds keys rotated at old_pos0 + u (u = index in block) */
#define BA_REENC_ABSOLUTE 1 /* cache holds every token of the block at old_pos0             */

typedef struct ba_tensor {
  void *ptr;           /* device pointer to element (token 0, head 0, dim 0) */
  int64_t stride_tok;  /* elements between consecutive tokens               */
  int64_t stride_head; /* elements between consecutive heads                */
  int32_t dtype;       /* BA_DTYPE_*                                        */
} ba_tensor;

typedef struct ba_heads {
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  const int32_t *q_to_kv; /* host, nullable -> h / (n_q_heads / n_kv_heads)             */
  float softmax_scale;    /* <= 0 -> 1 / sqrt(head_dim)                                 */
  double rope_base;       /* theta_j = rope_base^(-2j/head_dim) (Eq. 1's theta_j)       */
  const double *inv_freq; /* host, nullable: head_dim/2 overrides of theta_j            */
  int32_t rope_layout;    /* BA_ROPE_INTERLEAVED or BA_ROPE_HALF                        */
  const float *xcd_speed; /* host, nullable: relative speed of the device's 8 XCDs under the
                             attention core's load, from ba_measure_xcd_speed().  The final-block
                             calls then size their KV splits by the speed of the XCD each one
                             runs on, and choose which XCDs share KV heads (the XCDs of one
                             MI355X sustain clocks several per cent apart, and a launch ends with
                             its slowest workgroup).  Changes which
                             keys a split covers, hence low-order bits of the result, never the
                             workspace size.  null = equal splits.                             */
} ba_heads;

/* Library version (major * 10000 + minor * 100 + patch). */
int32_t ba_version(void);
/* Static name of a status code. */
const char *ba_status_string(int32_t status);
/* Thread-local text describing the last non-OK status returned on this thread. */
const char *ba_last_error(void);

/*
 * Relative speed of the eight XCDs of the current device under the attention core's load, for
 * ba_heads.xcd_speed (Section 2.5's step is the one whose launch ends with its slowest workgroup).
 * Runs the final-block attention core a few times on synthetic keys in the workspace (one workgroup
 * per compute unit, each timing its walk with the shader-clock and real-time counters), waits for
 * the stream, and writes eight numbers with mean 1: the share of the keys each XCD's split should get
 * for all of them to end together (a second pass with splits sized by the first pass's figures
 * corrects them).  If the device does not deal workgroups to XCDs round-robin as the planner
 * assumes, all eight are 1.
 * ws: 256-byte aligned, at least ba_measure_xcd_speed_workspace_bytes() bytes (about 150 MB).
 * Synchronises the stream; a one-time calibration, not a hot-path call.
 */
int32_t ba_measure_xcd_speed(float speed_out[8], void *ws, size_t ws_bytes, void *stream);
size_t ba_measure_xcd_speed_workspace_bytes(void);

/*
 * Diagnostic for benchmarks: where the time of one launch of the final-block attention core goes
 * (Section 2.5's step at 256 query tokens over 31,744 context tokens, 32 / 8 heads of 128: one
 * workgroup per compute unit, 8 KV splits of 62 or 63 key tiles).  The same synthetic run as
 * ba_measure_xcd_speed, same workspace; wave 0 of every workgroup reads the 100 MHz real-time counter
 * at its phase boundaries (means over four launches, after three that bring the clocks to their
 * steady state).  xcd_speed: host, nullable: eight figures as in ba_heads.xcd_speed, the
 * splits of the timed launch are sized by them (null: equal splits).
 * phases_us, microseconds, means over the workgroups unless noted:
 *   [0] kernel entry (first arguments loaded) -> first three tile copies issued
 *   [1] -> those tiles and the query fragments have landed
 *   [2] -> first scores done, the loop is entered (pipeline fill)
 *   [3] the walk over the key tiles
 *   [4] walk's end -> the split partial's stores complete
 *   [5] workgroup lifetime ([0] to [4] together)
 *   [6] first workgroup's entry -> last workgroup's stores complete (one number: the launch)
 *   [7] the longest walk of any workgroup (one number; [7] - [3] = what imbalance costs)
 * Synchronises the stream.  BA_ERR_UNSUPPORTED if the device does not give the probe's launch shape.
 */
#define BA_DIAG_PHASES 8
int32_t ba_diag_final_block_phases(double phases_us[BA_DIAG_PHASES], const float *xcd_speed, void *ws, size_t ws_bytes,
                                   void *stream);

/*
 * Diagnostic for benchmarks: the rate of v_mfma_f32_32x32x16_bf16 this device sustains on operands
 * with the bit activity of real data, 8 waves per compute unit, with 0, 1 or 2 one-KB operand
 * fragments re-read from LDS per two MFMAs (the attention core reads one per MFMA): the ceiling an
 * MFMA loop of that shape runs under when the part is power-limited, to set beside the nominal peak.
 * Runs for a few milliseconds and synchronises the stream.  Writes (each nullable) the TFLOP/s, the
 * shader clock sustained (GHz) and the fraction of cycles the matrix pipes were busy.
 * ws: 256-byte aligned, at least ba_diag_mfma_ceiling_workspace_bytes() bytes.
 */
int32_t ba_diag_mfma_ceiling(int32_t lds_reads_per_two_mfma, double *tflops, double *clock_ghz,
                             double *pipe_busy, void *ws, size_t ws_bytes, void *stream);
size_t ba_diag_mfma_ceiling_workspace_bytes(void);

/*
 * Per-kernel timing for benchmarks.  Between ba_profile_begin() and ba_profile_end() every
 * kernel launch the library makes is bracketed by two HIP events recorded on the launch
 * stream (at most max_records launches per class; later ones go untimed).
 * ba_profile_end() waits for the recorded events, writes per class the summed kernel time
 * in milliseconds and the number of timed launches (arrays of BA_PROFILE_CLASSES entries,
 * either may be null), frees the events and turns profiling off.  The events cost a few
 * microseconds per launch, so do not quote throughput from a profiled region.
 */
#define BA_PROFILE_ATTENTION 0 /* the MFMA attention core (encode and final block) */
#define BA_PROFILE_REENCODE 1  /* the RoPE rotation pass                            */
#define BA_PROFILE_COMBINE 2   /* the split-KV merge                                */
#define BA_PROFILE_CLASSES 3
int32_t ba_profile_begin(int32_t max_records);
int32_t ba_profile_end(double *ms_sum, int32_t *launches);

/*
 * Step 1 -- independent per-block causal attention (Section 1, step 1; Section 2.1).
 *
 * Token t of block b attends to tokens [c[b], t] of its own block only:
 *   o[t, h] = softmax_s(scale * <q^[t,h], k^[s,kv(h)]>) v[s, kv(h)],  s in [c[b], t].
 * q [T, n_q_heads, D], k, v [T, n_kv_heads, D], o [T, n_q_heads, D], all bf16.
 * block_offsets: host, n_blocks+1 ints, c[0] = 0 <= c[1] <= ... <= c[n_blocks] = T.
 * Blocks are independent, so a batch of prompts is simply a longer block list.
 * rope_mode BA_ROPE_APPLY rotates q and k at LOCAL positions (t - c[b]); then the
 * rotated keys -- the cacheable K of Section 2.3 -- are written to k_local_out
 * [T, n_kv_heads, D] if it is non-null, else kept in the workspace.  With
 * BA_ROPE_NONE k is used as given and k_local_out must be null.
 * Zero-length blocks are legal no-ops.  ws/ws_bytes: 256-byte aligned device workspace
 * of at least ba_encode_blocks_workspace_bytes() bytes (may be null when that is 0; with
 * BA_ROPE_APPLY it holds a table of rotation factors, and the rotated keys if k_local_out is null).
 */
int32_t ba_encode_blocks(const ba_heads *heads, const ba_tensor *q, const ba_tensor *k,
                         const ba_tensor *v, const ba_tensor *o_out,
                         const ba_tensor *k_local_out, int32_t n_blocks,
                         const int32_t *block_offsets, int32_t rope_mode, void *ws,
                         size_t ws_bytes, void *stream);
size_t ba_encode_blocks_workspace_bytes(const ba_heads *heads, int32_t n_blocks,
                                        const int32_t *block_offsets, int32_t rope_mode,
                                        int32_t have_k_local_out);

/*
 * Step 2 -- position re-encoding of cached keys (Section 2.3, Eq. 2 then Eq. 3).
 *
 * For block b and in-block index u, every layer and KV head:
 *   k' = R(p_new) R(p_old)^T k,  p_new = new_pos0[b] + u,
 *   p_old = old_pos0[b] + u (BA_REENC_SHIFT: a uniform rotation by new_pos0 - old_pos0)
 *        or old_pos0[b]     (BA_REENC_ABSOLUTE: e.g. a cache of un-rotated keys).
 * k_src / k_dst: [n_layers][tokens][n_kv_heads][D] with layer strides in elements; block
 * b is read from token src_tok_off[b] and written to token dst_tok_off[b] (a gather
 * into the prompt's K buffer).  k_dst may be exactly k_src (same pointer, strides and
 * offsets: in place); any other overlap is an error.  dtype bf16 (fp32 rotate, one
 * round-to-nearest-even on store) or fp32.  old_pos0 null -> 0; new_pos0 null ->
 * dst_tok_off.  A zero shift copies bit for bit.  Only heads->n_kv_heads, head_dim,
 * rope_base / inv_freq and rope_layout are read from `heads`.
 */
int32_t ba_reencode_positions(const ba_heads *heads, const ba_tensor *k_src,
                              const ba_tensor *k_dst, int32_t n_layers,
                              int64_t layer_stride_src, int64_t layer_stride_dst,
                              int32_t n_blocks, const int32_t *src_tok_off,
                              const int32_t *dst_tok_off, const int32_t *len,
                              const int32_t *old_pos0, const int32_t *new_pos0, int32_t mode,
                              void *stream);

/*
 * Step 3 -- final-block attention (Section 1, step 3; Section 2.5).
 *
 * Prompt n owns rows [cu_q[n], cu_q[n+1]) of q_f / k_f / v_f / o_out (its final block,
 * at least one token; cu_q[0] = 0) and rows [cu_ctx[n], cu_ctx[n+1]) of k_ctx / v_ctx (the
 * concatenated, already re-encoded KV of its earlier blocks; may be empty, then this is
 * plain causal attention).  Final-block token i attends to all context keys and to
 * final-block keys <= i.  Token i sits at absolute position q_pos0[n] + i (q_pos0 null ->
 * the prompt's context length).  With BA_ROPE_APPLY q_f and k_f are rotated at those
 * positions inside; k_ctx is always used as given.  k_f_rot_out (nullable, shaped like
 * k_f) receives the rotated final-block keys for later decoding.
 * All tensors bf16.  ws: 256-byte aligned, at least
 * ba_final_block_attention_workspace_bytes() bytes (rotated q_f and k_f, split partials).
 */
int32_t ba_final_block_attention(const ba_heads *heads, const ba_tensor *q_f,
                                 const ba_tensor *k_ctx, const ba_tensor *v_ctx,
                                 const ba_tensor *k_f, const ba_tensor *v_f,
                                 const ba_tensor *o_out, const ba_tensor *k_f_rot_out,
                                 int32_t n_prompts, const int32_t *cu_q, const int32_t *cu_ctx,
                                 const int32_t *q_pos0, int32_t rope_mode, void *ws,
                                 size_t ws_bytes, void *stream);
size_t ba_final_block_attention_workspace_bytes(const ba_heads *heads, int32_t n_prompts,
                                                const int32_t *cu_q, const int32_t *cu_ctx,
                                                int32_t rope_mode, int32_t have_k_f_rot_out);

/*
 * ba_final_block_attention for callers that cannot allocate device memory or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without ws / ws_bytes), same kernels and bit-identical results; the workspace is a
 * file-scope device array of BA_STATIC_SCRATCH_BYTES bytes that every GPU the library runs on holds
 * until the process ends.  The call allocates nothing on the device and frees nothing.  A call whose
 * ba_final_block_attention_workspace_bytes() exceeds BA_STATIC_SCRATCH_BYTES returns
 * BA_ERR_WORKSPACE and launches nothing.  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU (two streams, two threads) race; calls on one stream are safe.
 * Nothing in the array has to be cleared between calls: a call writes every byte it later reads.
 */
#define BA_STATIC_SCRATCH_BYTES (32u << 20)
int32_t ba_final_block_attention_static(const ba_heads *heads, const ba_tensor *q_f,
                                        const ba_tensor *k_ctx, const ba_tensor *v_ctx,
                                        const ba_tensor *k_f, const ba_tensor *v_f,
                                        const ba_tensor *o_out, const ba_tensor *k_f_rot_out,
                                        int32_t n_prompts, const int32_t *cu_q,
                                        const int32_t *cu_ctx, const int32_t *q_pos0,
                                        int32_t rope_mode, void *stream);

/*
 * Steps 2 and 3 in one call -- final-block attention straight from the block cache
 * (Section 2.3, Eq. 2 and 3; Section 2.5).
 *
 * Same result as ba_reencode_positions (BA_REENC_SHIFT) followed by ba_final_block_attention
 * with BA_ROPE_APPLY, but the cached keys are never rewritten: block b of a prompt stays at
 * the positions it was encoded at, and because a rotation of the key by the block's shift
 * equals a rotation of the query by minus that shift (the score only depends on the position
 * difference), the kernel turns its query fragments back once per block instead.  Many
 * prompts can therefore attend to one cached copy of a block at different offsets.
 *
 * Prompt n owns rows [cu_q[n], cu_q[n+1]) of q_f / k_f / v_f / o_out (cu_q[0] = 0, at least one
 * token) and blocks [cu_blk[n], cu_blk[n+1]) of the block table (cu_blk[0] = 0), in prompt
 * order.  Block b is rows [blk_tok_off[b], blk_tok_off[b] + blk_len[b]) of k_cache / v_cache
 * ([cache tokens, n_kv_heads, D], bf16); its keys carry the rotation of positions
 * blk_old_pos0[b] + u (null -> 0, the paper's local positions); in this prompt it sits at
 * positions blk_new_pos0[b] + u (null -> the total length of the prompt's earlier blocks).
 * Final-block token i sits at q_pos0[n] + i (null -> the prompt's context length); q_f and k_f
 * are un-rotated and are rotated inside; k_f_rot_out (nullable) receives the rotated k_f.
 * Empty blocks are skipped.
 *
 * gather_below: reading the block table in the kernel costs a fixed amount per block, a gathered
 * copy of the context an amount per token; when the mean length of the call's non-empty blocks is
 * below this many tokens (BA_GATHER_DEFAULT = 256 tokens; 0 = never gather) the call gathers the
 * context into its workspace first (keys re-encoded on the way, values copied; the cache itself
 * stays as it is) and continues as ba_final_block_attention.  Same results either way, to
 * rounding.  The two routes need different workspaces: pass the same value to the size query.
 * At most 1024 non-empty blocks per prompt when the kernel reads the block table
 * (BA_ERR_UNSUPPORTED beyond); no such limit on the gathered route.
 * All arrays host; ws: 256-byte aligned, at least
 * ba_final_block_attention_cached_workspace_bytes() bytes for the same gather_below.
 */
#define BA_GATHER_DEFAULT (-1)
int32_t ba_final_block_attention_cached(const ba_heads *heads, const ba_tensor *q_f,
                                        const ba_tensor *k_cache, const ba_tensor *v_cache,
                                        const ba_tensor *k_f, const ba_tensor *v_f,
                                        const ba_tensor *o_out, const ba_tensor *k_f_rot_out,
                                        int32_t n_prompts, const int32_t *cu_q,
                                        const int32_t *cu_blk, const int32_t *blk_tok_off,
                                        const int32_t *blk_len, const int32_t *blk_old_pos0,
                                        const int32_t *blk_new_pos0, const int32_t *q_pos0,
                                        int32_t gather_below, void *ws, size_t ws_bytes,
                                        void *stream);
size_t ba_final_block_attention_cached_workspace_bytes(const ba_heads *heads, int32_t n_prompts,
                                                       const int32_t *cu_q, const int32_t *cu_blk,
                                                       const int32_t *blk_len,
                                                       int32_t have_k_f_rot_out,
                                                       int32_t gather_below);

/*
 * Whole prompts in one call -- the attention mask of Section 2.4 (what a block fine-tune step
 * runs forward): the lower-triangular mask, cut so that a token sees its own block only, except
 * the tokens of a prompt's LAST block, which see every earlier token of the prompt.
 *
 * Prompt n owns blocks [cu_blk[n], cu_blk[n+1]) (cu_blk[0] = 0, at least one block each; the last
 * one is the block that sees the others); block b is tokens [block_offsets[b], block_offsets[b+1])
 * of q / k / v / o_out ([T, heads, D], bf16; block_offsets[0] = 0, non-decreasing, prompts packed
 * back to back).  With BA_ROPE_APPLY q and k are rotated inside at the token's position in its
 * prompt (first token of a prompt at 0) -- by Eq. 1's relative-position property the same scores
 * as local positions plus re-encoding -- and the rotated keys go to k_rot_out if non-null; with
 * BA_ROPE_NONE q and k are used as given.  lse_out (device, nullable): [T][n_q_heads] floats, the
 * natural-log sum of exp(scale * <q^, k^>) over each row's visible keys, as a backward pass needs.
 * Built for training-sized prompts: every row tile walks its key range alone (no KV splits), so a
 * short last block behind tens of thousands of context tokens is better served by
 * ba_final_block_attention.  The schedule packs the query heads of a KV head next to each other and
 * is laid out for groups of four or more; a smaller group (down to one query head per KV head) is
 * run as a group of four with zero phantom heads, through padded copies of q and o in the workspace
 * (correct, at up to four times the attention work).
 * ws: 256-byte aligned, at least ba_block_attention_prompts_workspace_bytes() bytes.
 */
int32_t ba_block_attention_prompts(const ba_heads *heads, const ba_tensor *q, const ba_tensor *k,
                                   const ba_tensor *v, const ba_tensor *o_out,
                                   const ba_tensor *k_rot_out, float *lse_out, int32_t n_prompts,
                                   const int32_t *cu_blk, const int32_t *block_offsets,
                                   int32_t rope_mode, void *ws, size_t ws_bytes, void *stream);
size_t ba_block_attention_prompts_workspace_bytes(const ba_heads *heads, int32_t n_prompts,
                                                  const int32_t *cu_blk,
                                                  const int32_t *block_offsets, int32_t rope_mode,
                                                  int32_t have_k_rot_out);

/*
 * Backward pass of ba_block_attention_prompts (rope_mode BA_ROPE_APPLY): given the gradient d_out
 * of the output, the gradients of the un-rotated q, k and v under the mask of Section 2.4.  With P
 * the masked softmax of the scaled scores of the rotated q^ and k^:
 *   dV = P^T dO,  dS = P o (dO V^T - rowsum(dO o O)),  dq^ = scale * dS k^,  dk^ = scale * dS^T q^,
 * and dq, dk are dq^, dk^ turned back by the rotation of Eq. 1 (an orthogonal map).  Query heads
 * that share a KV head add up in dk and dv.  P is recomputed from q, k and the rows' log-sum-exps;
 * nothing else of the forward pass is kept.
 *
 * q, k, v, cu_blk, block_offsets: as given to the forward call.  o [T, n_q_heads, D] and lse
 * (device, [T][n_q_heads] floats): its outputs.  d_out [T, n_q_heads, D]; dq_out like q, dk_out and
 * dv_out like k and v; all bf16, fully overwritten.  Deterministic: every sum has one owner, no
 * atomics.  Fewer than four query heads per KV head: run as groups of four, as in the forward call
 * (phantom heads have a zero output gradient and add nothing to dk and dv).  ws: 256-byte aligned, at least
 * ba_block_attention_prompts_backward_workspace_bytes() bytes.
 */
int32_t ba_block_attention_prompts_backward(const ba_heads *heads, const ba_tensor *q,
                                            const ba_tensor *k, const ba_tensor *v,
                                            const ba_tensor *o, const float *lse,
                                            const ba_tensor *d_out, const ba_tensor *dq_out,
                                            const ba_tensor *dk_out, const ba_tensor *dv_out,
                                            int32_t n_prompts, const int32_t *cu_blk,
                                            const int32_t *block_offsets, void *ws,
                                            size_t ws_bytes, void *stream);
size_t ba_block_attention_prompts_backward_workspace_bytes(const ba_heads *heads,
                                                           int32_t n_prompts,
                                                           const int32_t *cu_blk,
                                                           const int32_t *block_offsets);

/*
 * The schedule of a call, for inspection and tests: the work items the host planner hands to the
 * kernels, computed by the code the calls themselves use.  Host only: no device is touched, so
 * these run on a machine without a GPU.
 *
 * A work item is one workgroup's job at one KV head (an item with kv_head = -1 runs once per KV
 * head; with splits sized by XCD speed the final-block query lists every KV head's items): packed query
 * rows [row_begin, row_end) of a "problem" (row = token_in_problem * group + head_in_group, group =
 * n_q_heads / n_kv_heads) against two key ranges -- context keys [ctx_begin, ctx_end), counted from
 * the problem's first visible context key and all visible to every row, and the problem's own
 * tokens [self_begin, self_end) as keys, of which token i sees those <= i (Section 2.1's causal
 * block; Section 2.5's final block; Section 2.4's mask for whole prompts).  Key ranges are whole
 * key tiles of tile_keys keys, cut at the end of the segment.  Items of one (problem, row range)
 * that differ in `split` are merged by the split merge.
 * Each query returns the number of items (also when `items` is null or max_items is smaller: then
 * only the first max_items are written), or a negative BA_ERR_* status.
 */
typedef struct ba_work_item {
  int32_t launch;      /* which kernel launch of the call                                       */
  int32_t problem;     /* prompt (final block, whole prompts) or block (per-block encoding)     */
  int32_t first_token; /* row of q / o that is the problem's token 0                            */
  int32_t tile_rows, tile_keys;
  int32_t row_begin, row_end;
  int32_t split, n_splits;
  int32_t ctx_begin, ctx_end;
  int32_t self_begin, self_end;
  int32_t kv_head;     /* the KV head, or -1: the same item at every KV head                    */
  int32_t xcd;         /* with kv_head >= 0: the XCD (of eight) whose compute units run it, else -1 */
} ba_work_item;
/* ba_final_block_attention on a device of n_compute_units compute units (256 on MI355X). */
int64_t ba_schedule_final_block(const ba_heads *heads, int32_t n_prompts, const int32_t *cu_q,
                                const int32_t *cu_ctx, int32_t n_compute_units,
                                ba_work_item *items, int64_t max_items);
/* ba_encode_blocks with packed tensors ([tokens][heads][head_dim]). */
int64_t ba_schedule_encode_blocks(const ba_heads *heads, int32_t n_blocks,
                                  const int32_t *block_offsets, ba_work_item *items,
                                  int64_t max_items);
/* ba_block_attention_prompts: `problem` is the prompt, first_token the block's first token; the
 * context range counts from the first token of the prompt (a passage block has none). */
int64_t ba_schedule_prompts(const ba_heads *heads, int32_t n_prompts, const int32_t *cu_blk,
                            const int32_t *block_offsets, ba_work_item *items, int64_t max_items);

#ifdef __cplusplus
}
#endif
#endif /* BA_H_ */
