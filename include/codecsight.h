/*
 * codecsight.h -- C ABI of the codec-guided sliding-window prefill hot path
 * (CodecSight, arXiv 2604.06036) for AMD MI355X (gfx950 / CDNA4).
 *
 * One slide step of one batch of video streams runs, in this order:
 *
 *   cs_score_compact        once     codec metadata -> keep mask -> ordered kept-token list
 *   cs_kv_rerotate          once     reused cached keys: RoPE correction by the position shift,
 *                                    all decoder layers in one launch (values copied when repacking)
 *   for each decoder layer:
 *     cs_kv_refresh_scatter          freshly computed K/V rows of refresh + new tokens -> cache
 *     cs_window_prefill_attn         causal GQA attention of those tokens over the mixed cache
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Every pointer argument is a DEVICE pointer owned by the caller, except `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream).  The library allocates
 *    nothing, keeps no per-call state, never synchronises, and enqueues all work on `stream`.
 *  - Scalars are host values.  Strides are in ELEMENTS of the cache dtype.
 *  - Return value: CS_OK, or a negative CS_E* code.  Argument errors are detected on the host
 *    before anything is launched, so a failed call has no side effects on device memory.
 *  - A cache "slot" is a row index into the KV pool: slot = block_id * 16 + offset_in_block.
 *    The pool of one layer is addressed as  base + slot*stride_slot + kv_head*stride_head + c.
 *  - dtype: CS_F32 (float) or CS_BF16 (bfloat16 bit patterns, uint16_t storage).
 *  - Not checked on the device (caller's contract): slots lie inside the pool; destination
 *    slots are unique; for a repacking re-rotation the source and destination slot sets are
 *    disjoint; q_pos is non-decreasing inside a stream and smaller than that stream's kv_len.
 */
#ifndef CODECSIGHT_H_
#define CODECSIGHT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CS_OK            0
#define CS_EINVAL       (-1)  /* null / negative / inconsistent argument                        */
#define CS_EUNSUPPORTED (-2)  /* dtype, head_dim, block size, group, alignment outside support  */
#define CS_EHIP         (-3)  /* a HIP launch failed; cs_last_hip_error() holds the HIP code     */
#define CS_EWORKSPACE   (-4)  /* workspace missing, misaligned or smaller than *_workspace()     */

#define CS_F32  0
#define CS_BF16 1

#define CS_FRAME_P 0
#define CS_FRAME_I 1

#define CS_ROPE_HALF_SPLIT  0  /* pairs (i, i + d/2) */
#define CS_ROPE_INTERLEAVED 1  /* pairs (2i, 2i + 1) */

#define CS_KV_BLOCK 16         /* tokens per cache block */

/* cs_window_prefill_attn: what the workspace holds when the call starts */
#define CS_ATTN_PLAN_BUILD 0   /* nothing: plan the work from cu_q / q_pos, then run              */
#define CS_ATTN_PLAN_REUSE 1   /* the plan an earlier BUILD call left there (same workspace, same
                                  cu_q / q_pos / block_table contents and shape arguments):
                                  run straight away                                              */
#define CS_ATTN_PLAN_ONLY  2   /* nothing: plan the work and return without computing attention   */

/* Library identification, e.g. "codecsight-mi355x 0.1 (gfx950)". Static storage. */
const char* cs_version(void);

/* HIP error code (hipError_t as int) of the most recent CS_EHIP on the calling thread, else 0. */
int cs_last_hip_error(void);

/* ------------------------------------------------------------------------------------------
 * Measurement aid (no passage of the paper: it computes nothing of the method).  Launches
 * n_workgroups workgroups of 256 threads that each issue iters * 8 v_mfma_f32_32x32x16_bf16 per wave
 * on register operands (constant ones, or lane-dependent pseudo-random ones when random_operands
 * != 0) and store nothing; 4 waves * iters * 8 * 32768 flop per workgroup.  bench.py times it to
 * report the bf16 matrix-core rate this device sustains, beside the published peak.
 *  sink  device float [n_workgroups * 256], never written in practice
 * Errors: CS_EINVAL (null sink, n_workgroups or iters < 1, n_workgroups > 2^20), CS_EHIP.
 * ------------------------------------------------------------------------------------------ */
int cs_mfma_rate_probe(float* sink, int32_t n_workgroups, int32_t iters, int32_t random_operands,
                       void* stream);

/* ------------------------------------------------------------------------------------------
 * (m) Block-to-patch projection.     Paper Sec. 3.3.1, paragraph on mapping codec changes to ViT
 *     patches: block rectangles live in source-frame pixels, patches in model-input pixels; the
 *     rectangles are rescaled and every patch is given the strongest motion (Eq. 1) found among
 *     the blocks that land on it.  Sec. 3.3.2: a patch touched by an intra-coded block is kept.
 *     Produces the `mv` and `intra` inputs of cs_score_compact from a decoder's per-block output.
 *
 * Block m covers source pixels [x, x+w) x [y, y+h), clipped to the src_w x src_h frame; its image
 * is [x sx, (x+w) sx) x [y sy, (y+h) sy) with sx = in_w/src_w, sy = in_h/src_h (a plain resize).
 * Patch (r, c) of the grid_h x grid_w grid is [c patch, (c+1) patch) x [r patch, (r+1) patch) in
 * input pixels; "overlap" is an intersection of positive area, decided in exact integer
 * arithmetic.  Per frame f and patch i = r*grid_w + c:
 *     mv[f][i]    = (dx, dy) of the overlapping inter block with the largest dx^2 + dy^2, ties to
 *                   the lexicographically largest (dx, dy) (so block order never matters);
 *                   (0, 0) when no inter block overlaps
 *     intra[f][i] = 1 if a block with CS_BLOCK_INTRA overlaps, else 0 (such blocks carry no vector
 *                   and take no part in the maximum)
 *
 *  blocks      in   cs_block [cu_blocks[n_frames]], 16-byte aligned; frame f owns records
 *                   cu_blocks[f] .. cu_blocks[f+1]-1, in any order
 *  cu_blocks   in   int32 [n_frames+1], non-decreasing
 *  mv          out  int16 [n_frames][grid_h*grid_w][2], 4-byte aligned;  intra  out  uint8 [n_frames][grid_h*grid_w]
 * All pointers are device memory.  Bit exact (integer work).
 * Errors: CS_EINVAL (null pointer, negative n_frames, a size < 1), CS_EUNSUPPORTED (a frame or
 *         input dimension > 16384, patch > 1024, grid_h*grid_w > 7168, misaligned blocks / mv),
 *         CS_EHIP.  n_frames == 0 returns CS_OK.
 * ------------------------------------------------------------------------------------------ */
#define CS_BLOCK_INTRA 1u      /* cs_block.flags bit 0: intra-coded, dx/dy meaningless */

typedef struct cs_block {
  uint16_t x, y;               /* top-left corner, source-frame pixels */
  uint16_t w, h;               /* size, source-frame pixels            */
  int16_t dx, dy;              /* motion vector (any fixed unit, e.g. quarter pel) */
  uint32_t flags;
} cs_block;

int cs_project_blocks(const cs_block* blocks, const int32_t* cu_blocks, int32_t n_frames,
                      int32_t src_w, int32_t src_h, int32_t in_w, int32_t in_h, int32_t patch,
                      int32_t grid_h, int32_t grid_w, int16_t* mv, uint8_t* intra, void* stream);

/* ------------------------------------------------------------------------------------------
 * (r) Residual proxy.     Paper Sec. 4, "Codec Processing" (the decoder exposes no prediction
 *     residuals; a patch is scored by how far its pixels are, on average and in absolute value,
 *     from the previous decoded frame displaced by the motion vectors); it stands in for the block
 *     residual of Eq. 2 and feeds the rescue rule of Eq. 4.  Produces the `sad` input of
 *     cs_score_compact.
 *
 * Frames are 8-bit luma planes at source resolution.  The motion field holds one quarter-pixel
 * vector (dx, dy) per cell x cell pixel cell (intra cells: (0, 0)).  For pixel (x, y) of frame f:
 *     (ox, oy)   = (floor((dx + 2) / 4), floor((dy + 2) / 4))        whole-pixel vector
 *     pred(x, y) = prev[f][clamp(y + oy, 0, src_h-1)][clamp(x + ox, 0, src_w-1)]
 * The pixel belongs to patch column floor(x * in_w / (patch * src_w)) and row
 * floor(y * in_h / (patch * src_h)) (the plain resize of cs_project_blocks); pixels outside the
 * grid_h x grid_w grid are ignored.  Per patch i with n_i pixels:
 *     res[f][i] = floor(256 * sum |cur - pred| / n_i)      (1/256 grey levels; 0 when n_i = 0)
 *
 *  cur, prev   in   uint8, frame f at + f*frame_stride, row y at + y*pitch (bytes); 16-byte aligned
 *  mv_field    in   int16 [n_frames][ceil(src_h/cell)][ceil(src_w/cell)][2], 4-byte aligned
 *  res         out  uint32 [n_frames][grid_h*grid_w], 4-byte aligned (also the accumulator: the
 *                   call clears it first)
 * All pointers are device memory.  Bit exact (integer work).
 * Errors: CS_EINVAL (null pointer, negative n_frames, a size < 1, pitch < src_w, frame_stride <
 *         pitch*src_h), CS_EUNSUPPORTED (cell not 4, 8 or 16; a frame or input dimension > 16384;
 *         patch > 1024; grid_w > 8192; pitch or frame_stride not a multiple of 16, pitch below
 *         src_w rounded up to 16; misaligned pointers; patch columns narrower than 4 source
 *         pixels, i.e. patch*src_w < 4*in_w), CS_EHIP.  n_frames == 0 returns CS_OK.
 * ------------------------------------------------------------------------------------------ */
int cs_residual_proxy(const uint8_t* cur, const uint8_t* prev, const int16_t* mv_field,
                      int32_t n_frames, int32_t src_w, int32_t src_h, int64_t pitch,
                      int64_t frame_stride, int32_t cell, int32_t in_w, int32_t in_h, int32_t patch,
                      int32_t grid_h, int32_t grid_w, uint32_t* res, void* stream);

/* ------------------------------------------------------------------------------------------
 * (a) Change scoring + ordered token compaction.       Paper Sec. 3.3.1-3.3.2, Eq. 1, 3, 4, 5,
 *     "Temporal stabilization within a GOP", "Adapting sparsity to the model layout".
 *
 * The batch holds n_frames frames of n_streams streams; stream s owns frames
 * cu_frames[s] .. cu_frames[s+1]-1 (temporal order).  Each frame has P = grid_h*grid_w patches
 * (row-major) and T = (grid_h/group)*(grid_w/group) visual tokens (row-major token grid).
 *
 * Per stream, frames are visited in temporal order:
 *   I-frame : every token is kept; the accumulated mask is reset to zero; the frame's metadata
 *             is not read (an I-frame carries no inter-frame motion vectors).
 *   P-frame : for patch i,  m = dx*dx + dy*dy  (integers, no rounding anywhere)
 *               d_mv  = m >= tau_mv_sq                              (Eq. 3, squared)
 *               d_res = use_residual && !d_mv && sad[i] >= tau_sad   (Eq. 4)
 *               d     = d_mv | d_res | (intra && intra[i] != 0)      (Eq. 5)
 *             acc[i] |= d (GOP accumulation; with acc_mask == NULL the patch mask is d itself),
 *             a token is kept when any patch of its group x group block is selected.
 * Kept tokens of all frames are then listed in frame-major, row-major order (the selection keeps
 * the tokens' original relative order, Sec. 3.3.2).
 *
 * Thresholds are integers in the metadata's own units, so the mask is exact: a threshold of
 * tau pixels on quarter-pel vectors is tau_mv_sq = (4*tau)^2; a strict '>' is '>= value+1'.
 *
 *  mv         in   int16  [n_frames][P][2]   (dx, dy), 4-byte aligned
 *  sad        in   uint32 [n_frames][P]      NULL iff use_residual == 0
 *  intra      in   uint8  [n_frames][P]      nullable: non-zero = patch overlaps an intra block
 *  frame_type in   uint8  [n_frames]         CS_FRAME_P / CS_FRAME_I
 *  cu_frames  in   int32  [n_streams+1]      non-decreasing, cu_frames[0]=0, last = n_frames
 *  acc_mask   i/o  uint8  [n_streams][P]     nullable; 0/1 per patch; state carried across calls
 *  keep_mask  out  uint8  [n_frames][T]      0/1
 *  kept_idx   out  int32  [n_frames*T]       first kept_off[n_frames] entries valid: ids f*T+t,
 *                                            strictly ascending; the tail is left untouched
 *  kept_off   out  int32  [n_frames+1]       exclusive prefix of per-frame kept counts
 *  workspace       cs_score_compact_workspace() bytes, 8-byte aligned; contents need not be
 *                  initialised.  Two calls that overlap in time must not share a workspace.
 *                  After the call has completed on the stream, the 32-bit word at byte offset
 *                  CS_SCORE_STATUS_OFFSET of the workspace is the call's device status: 0, or 1
 *                  when a tile's wait for the kept-token count of its predecessors ran out (the
 *                  wait is bounded so that every wave exits; it expires only if a workgroup of the
 *                  launch never ran).  With status 1 kept_idx / kept_off are not valid.  The rest
 *                  of the workspace is meaningless afterwards.  The return value cannot carry this
 *                  (the call never synchronises): callers that must know read the word after
 *                  synchronising.
 * Errors: CS_EINVAL (null required pointer, n_streams < 0, n_frames < 0, grid < 1,
 *         grid not divisible by group, sad/use_residual mismatch), CS_EUNSUPPORTED (group not in
 *         {1,2}, n_frames*T >= 2^31), CS_EWORKSPACE, CS_EHIP.  n_streams == 0 or n_frames == 0
 *         writes kept_off[0..n_frames] = 0 and returns CS_OK.
 * ------------------------------------------------------------------------------------------ */
#define CS_SCORE_STATUS_OFFSET 4   /* byte offset of the device status word in the workspace */

size_t cs_score_compact_workspace(int32_t n_streams, int32_t n_frames,
                                  int32_t grid_h, int32_t grid_w, int32_t group);

int cs_score_compact(const int16_t* mv, const uint32_t* sad, const uint8_t* intra,
                     const uint8_t* frame_type, const int32_t* cu_frames, uint8_t* acc_mask,
                     int32_t n_streams, int32_t n_frames,
                     int32_t grid_h, int32_t grid_w, int32_t group,
                     uint32_t tau_mv_sq, uint32_t tau_sad, int32_t use_residual,
                     uint8_t* keep_mask, int32_t* kept_idx, int32_t* kept_off,
                     void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * (a') cs_score_compact for callers that cannot allocate device memory or pass a workspace: code
 *     under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 *
 * Same arguments, results and errors as cs_score_compact, without the workspace: the look-back words
 * live in an array the library holds in device memory of each GPU (8,448 bytes per GPU, kept until
 * the process ends).  Limit: n_streams <= 4096 (CS_EUNSUPPORTED beyond: use cs_score_compact).
 * The call allocates nothing and calls no allocating routine; its first call on a device looks up
 * the array's address (make that call outside a graph capture).  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (different streams) race and must be
 * serialised by the caller; back-to-back calls on one stream are fine (each call clears what it
 * needs with a kernel of its own, whatever the previous call left).  The device status word
 * described above is not readable through this entry point.
 * ------------------------------------------------------------------------------------------ */
int cs_score_compact_noalloc(const int16_t* mv, const uint32_t* sad, const uint8_t* intra,
                             const uint8_t* frame_type, const int32_t* cu_frames, uint8_t* acc_mask,
                             int32_t n_streams, int32_t n_frames,
                             int32_t grid_h, int32_t grid_w, int32_t group,
                             uint32_t tau_mv_sq, uint32_t tau_sad, int32_t use_residual,
                             uint8_t* keep_mask, int32_t* kept_idx, int32_t* kept_off, void* stream);

/* ------------------------------------------------------------------------------------------
 * (p) Refresh plan on the device.     Paper Sec. 3.4.1 (overlap I-frames are anchors and are
 *     recomputed, the other overlap frames reuse their cached K/V, new frames and the text
 *     suffix are prefilled) and Sec. 3.5 (planning precedes KV-context preparation; a frame-aware
 *     index maps visual-token spans to physical cache slots across cache-block boundaries).
 *
 * All n_streams windows advance by `stride` frames.  Per stream s the previous window held the
 * kept visual tokens of its `window` frames in frame order, then n_text text tokens, entry j of
 * that sequence in slot  block_table_old[s][j/16]*16 + j%16.  The new window is frames
 * stride .. window-1 of the old one (the overlap) followed by the `stride` new frames, whose
 * kept-token counts are kept_off[s*stride+f+1] - kept_off[s*stride+f] (cs_score_compact's
 * output for a batch of `stride` frames per stream, stream-major), then the text; its entry j
 * lives in slot  block_table_new[s][j/16]*16 + j%16.  Walking the new sequence in order:
 *   token of an overlap frame that is not an I-frame -> one reused row: src_slot (its slot in the
 *       old window), dst_slot (its slot in the new one), delta = -stride*tokens_per_frame
 *       (positions are dense: frame slot * tokens_per_frame + token id);
 *   token of an overlap I-frame (kind 0), of a new frame (kind 1), text token (kind 2)
 *       -> one executed row: q_pos = j, q_slot = its new slot, q_kind.
 * Reused rows of all streams are concatenated stream-major, and so are executed rows;
 * cu_q[s] .. cu_q[s+1]-1 are stream s's executed rows, kv_len[s] the new sequence length.
 * The lists are what cs_kv_rerotate (src_slot, dst_slot, delta), cs_kv_refresh_scatter (q_slot)
 * and cs_window_prefill_attn (cu_q, q_pos, kv_len, block_table_new) take; nothing returns to
 * the host.  Entries between a list's total and its capacity are padded (slots -1, which the
 * consumers skip, delta 0, q_pos 0, q_kind 0xff), so the consumers can be called with the
 * capacities as their row counts.
 *
 *  old_types, old_counts   in   uint8 / int32 [n_streams][window]   the cached window
 *  new_types               in   uint8 [n_streams][stride]
 *  kept_off                in   int32 [n_streams*stride + 1]
 *  block_table_old / _new  in   int32 [n_streams][max_blocks_old / _new]
 *  src_slot, dst_slot, delta    out  int32 [reuse_cap]
 *  q_pos, q_slot, q_kind        out  int32, int32, uint8 [q_cap]
 *  cu_q  out int32 [n_streams+1];  kv_len  out int32 [n_streams]
 *  out_types, out_counts   out  uint8 / int32 [n_streams][window]: the new window, the next
 *                          step's old_types / old_counts (must not alias them)
 *  totals                  out  int32 [4]: reused rows, executed rows, flags (1: reused rows exceed
 *                          reuse_cap, 2: executed rows exceed q_cap, 4: a sequence index falls
 *                          outside its block-table row), 0.  Rows beyond a capacity are not
 *                          written and cu_q is clamped to q_cap (the streams that do not fit lose
 *                          their last executed rows), so the consumers stay inside the lists
 *                          whatever the flags say; a row whose slot cannot be formed gets slot -1
 *                          (and an executed row's q_pos is pulled back to the last position its
 *                          block-table row covers, so attention never indexes past the table).
 *  workspace               cs_plan_refresh_workspace() bytes, 16-byte aligned, contents need not
 *                          be initialised
 * All pointers are device memory.  Bit exact (integer work).
 * Errors: CS_EINVAL (null pointer, negative size, window < 1, stride outside 1..window,
 *         tokens_per_frame < 1, a block table without columns), CS_EUNSUPPORTED
 *         (n_streams*(window+1), a capacity or stride*tokens_per_frame >= 2^31), CS_EWORKSPACE,
 *         CS_EHIP.
 * ------------------------------------------------------------------------------------------ */
size_t cs_plan_refresh_workspace(int32_t n_streams, int32_t window);

int cs_plan_refresh(const uint8_t* old_types, const int32_t* old_counts,
                    const uint8_t* new_types, const int32_t* kept_off,
                    const int32_t* block_table_old, int32_t max_blocks_old,
                    const int32_t* block_table_new, int32_t max_blocks_new,
                    int32_t n_streams, int32_t window, int32_t stride, int32_t n_text,
                    int32_t tokens_per_frame, int64_t reuse_cap, int64_t q_cap,
                    int32_t* src_slot, int32_t* dst_slot, int32_t* delta,
                    int32_t* q_pos, int32_t* q_slot, uint8_t* q_kind,
                    int32_t* cu_q, int32_t* kv_len, uint8_t* out_types, int32_t* out_counts,
                    int32_t* totals, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * (b) Position-corrected reuse of cached keys.          Paper Sec. 3.4.2, Eq. 6; Sec. 3.5
 *     (reusable states are repacked into the destination cache of the current request).
 *
 * For every reused row r, every layer l < n_layers and every kv head h:
 *     K[l][dst_slot[r]][h] = R(delta[r]) * K[l][src_slot[r]][h]
 * with the one-dimensional RoPE rotation  R(D): for pair (a, b) with frequency index i,
 *     theta_i = rope_base^(-2i/head_dim),  out_a = x_a cos(D theta_i) - x_b sin(D theta_i),
 *                                          out_b = x_b cos(D theta_i) + x_a sin(D theta_i),
 * (a, b) = (i, i + head_dim/2) for CS_ROPE_HALF_SPLIT, (2i, 2i+1) for CS_ROPE_INTERLEAVED.
 * delta = p_new - p_old, signed.  Angles are formed in double precision and reduced before
 * the single-precision sin/cos; products and the final rounding are single precision.
 * When dst_slot != NULL (repack) V[l][dst_slot[r]][h] = V[l][src_slot[r]][h] is copied bit for
 * bit (values carry no position).  When dst_slot == NULL the keys are rotated in place and
 * v_cache is not touched (may be NULL).
 *
 *  k_cache, v_cache  i/o  pool of all layers: element (l, slot, h, c) at
 *                         l*stride_layer + slot*stride_slot + h*stride_head + c; 16-byte aligned
 *  src_slot, delta   in   int32 [n_rows];   dst_slot in int32 [n_rows] or NULL; a row with a
 *                         negative src_slot or dst_slot is skipped
 * Errors: CS_EINVAL (null k_cache/src_slot/delta, v_cache NULL with dst_slot given, negative
 *         sizes, rope_base <= 0), CS_EUNSUPPORTED (head_dim not a multiple of 16 or > 256,
 *         strides not multiples of 16 bytes, unknown dtype / rope_style), CS_EHIP.
 *         n_rows == 0 returns CS_OK without a launch.
 * ------------------------------------------------------------------------------------------ */
int cs_kv_rerotate(void* k_cache, void* v_cache,
                   const int32_t* src_slot, const int32_t* dst_slot, const int32_t* delta,
                   int64_t n_rows, int32_t n_layers, int32_t n_kv_heads, int32_t head_dim,
                   int64_t stride_layer, int64_t stride_slot, int64_t stride_head,
                   float rope_base, int32_t rope_style, int32_t dtype, void* stream);

/* ------------------------------------------------------------------------------------------
 * (b') The same correction for multidimensional RoPE.       Paper Sec. 3.4.2 (after Eq. 6: with
 *     several positional components, each rotary dimension is corrected by the component the
 *     model maps to it); Sec. 4 names Qwen3-VL's three-axis mRoPE.
 *
 * A position is a triple (t, h, w).  Frequency pair i of a head (the same pairs and the same
 * theta_i = rope_base^(-2i/head_dim) as in cs_kv_rerotate) is driven by positional component
 * axis_of_pair[i], so row r rotates pair i by delta3[r][axis_of_pair[i]] * theta_i.  With every
 * pair on one axis this is cs_kv_rerotate of that component.
 *
 *  delta3        in   int32 [n_rows][3]   (d_t, d_h, d_w) = p_new - p_old per component
 *  axis_of_pair  in   uint8 [head_dim/2]  values 0, 1, 2 (a larger value is read as 2); device memory
 * All other arguments, layouts, aliasing rules and errors as for cs_kv_rerotate; CS_EINVAL also
 * when axis_of_pair is NULL.
 * ------------------------------------------------------------------------------------------ */
int cs_kv_rerotate_axes(void* k_cache, void* v_cache,
                        const int32_t* src_slot, const int32_t* dst_slot, const int32_t* delta3,
                        const uint8_t* axis_of_pair, int64_t n_rows,
                        int32_t n_layers, int32_t n_kv_heads, int32_t head_dim,
                        int64_t stride_layer, int64_t stride_slot, int64_t stride_head,
                        float rope_base, int32_t rope_style, int32_t dtype, void* stream);

/* ------------------------------------------------------------------------------------------
 * (c) In-place refresh write.                            Paper Sec. 3.5 (at each layer the K/V
 *     just computed go straight into the destination cache, before attention runs).
 *
 * One layer:  K[slot[i]][h] = k_new[i][h],  V[slot[i]][h] = v_new[i][h]  for slot[i] >= 0;
 * a negative slot skips the token.  Pure data movement, bit exact.
 *
 *  k_new, v_new       in   [n_tok][n_kv_heads][head_dim] contiguous, 16-byte aligned
 *  slot               in   int32 [n_tok]
 *  k_cache_layer, v_cache_layer  i/o  pool already offset to the layer, 16-byte aligned
 * Errors: CS_EINVAL (null pointer, negative size), CS_EUNSUPPORTED (row bytes or strides not a
 *         multiple of 16 bytes, unknown dtype), CS_EHIP.  n_tok == 0 returns CS_OK.
 * ------------------------------------------------------------------------------------------ */
int cs_kv_refresh_scatter(const void* k_new, const void* v_new, const int32_t* slot,
                          void* k_cache_layer, void* v_cache_layer,
                          int64_t n_tok, int32_t n_kv_heads, int32_t head_dim,
                          int64_t stride_slot, int64_t stride_head, int32_t dtype, void* stream);

/* ------------------------------------------------------------------------------------------
 * (d) Joint prefill attention of refresh + suffix tokens over the mixed cache.   Paper Sec. 3.5
 *     (attention reads reused states and states of the current pass side by side, so the suffix
 *     sees the refreshed anchors).
 *
 * One layer, n_streams streams in one variable-length launch.  Stream s owns query rows
 * cu_q[s] .. cu_q[s+1]-1; query t sits at window-sequence index q_pos[t] and sees cache entries
 * j = 0 .. q_pos[t] of its stream, entry j living in slot
 *     block_table[s*max_blocks + j/16] * 16 + j%16.
 * For query head h (kv head g = h / (n_q_heads / n_kv_heads)):
 *     out[t][h] = sum_j softmax_j(softmax_scale * q[t][h] . K[slot_j][g]) * V[slot_j][g]
 * Keys and queries arrive already rotated; no positional work happens here.
 * CS_BF16: bf16 operands on the matrix cores, fp32 scores / statistics / accumulation, bf16
 * result.  CS_F32: fp32 throughout.
 *
 *  q, out        [n_q][n_q_heads][head_dim] contiguous, 16-byte aligned
 *  cu_q          int32 [n_streams+1], cu_q[0] = 0, cu_q[n_streams] <= n_q: n_q sizes the launch
 *                and may be an upper bound (rows from cu_q[n_streams] on are neither read nor
 *                written), so that a plan made on the device needs no host copy of its totals
 *  q_pos         int32 [n_q], non-negative, non-decreasing inside a stream;  kv_len int32
 *                [n_streams]: block_table row s defines entries 0 .. ceil(kv_len[s]/16)-1.  A
 *                q_pos at or past kv_len[s] (or past max_blocks*16) is read as the last defined
 *                entry, so the call never indexes beyond the rows the table defines; the rows of
 *                a stream with kv_len <= 0 are not computed (their `out` rows stay untouched)
 *  block_table   int32 [n_streams][max_blocks]
 *  workspace     cs_window_prefill_attn_workspace() bytes for the same shape arguments, 16-byte
 *                aligned (may be 0, then NULL is accepted).  Holds the work plan of the launch
 *                (the list of (stream, kv head, row tile, key range) items each XCD serves, a
 *                function of cu_q, q_pos and block_table only) and the partial results of row
 *                tiles whose key sweep is shared by several items.  Two calls that overlap in
 *                time must not share a workspace.
 *  plan_mode     CS_ATTN_PLAN_BUILD: workspace contents need not be initialised; the call plans
 *                and runs.  CS_ATTN_PLAN_REUSE: the workspace still holds the plan of an earlier
 *                BUILD call with identical cu_q / q_pos / block_table contents and shape
 *                arguments (the decoder layers of one step: build at the first layer, reuse at
 *                the others); the planning launch is skipped.  CS_ATTN_PLAN_ONLY: plan and return
 *                (q, the caches and out are not touched and may be NULL), for callers that
 *                prefer every layer to run in REUSE mode.  Ignored where no plan is used (CS_F32, head_dim 64: an
 *                ONLY call then computes like any other).
 * Errors: CS_EINVAL (null pointer, negative size, n_q_heads not a multiple of n_kv_heads, unknown
 *         plan_mode, softmax_scale not a positive finite number), CS_EUNSUPPORTED (head_dim not in {64,128}, block_size != 16,
 *         n_q_heads/n_kv_heads > 16, strides not multiples of 16 bytes, unknown dtype; CS_BF16:
 *         n_kv_heads > 256, n_streams >= 2^23, stride_slot >= 2^26 elements or max_blocks >= 2^17
 *         with head_dim 128, max_blocks > 8192 with head_dim 64),
 *         CS_EWORKSPACE, CS_EHIP.
 *         n_q == 0 or n_streams == 0 returns CS_OK.
 * ------------------------------------------------------------------------------------------ */
size_t cs_window_prefill_attn_workspace(int64_t n_q, int32_t n_streams, int32_t n_q_heads,
                                        int32_t n_kv_heads, int32_t head_dim, int32_t max_blocks,
                                        int32_t dtype);

int cs_window_prefill_attn(const void* q, const void* k_cache_layer, const void* v_cache_layer,
                           const int32_t* cu_q, const int32_t* q_pos, const int32_t* kv_len,
                           const int32_t* block_table, int32_t max_blocks, int32_t block_size,
                           void* out, int64_t n_q, int32_t n_streams,
                           int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                           int64_t stride_slot, int64_t stride_head, float softmax_scale,
                           int32_t dtype, void* workspace, size_t workspace_bytes,
                           int32_t plan_mode, void* stream);

/* ------------------------------------------------------------------------------------------
 * (c+d) Refresh write and joint prefill attention as one call.        Paper Sec. 3.5: at each layer
 *     the K/V just computed for the refresh and suffix tokens are written straight into the
 *     destination cache, ahead of that layer's causal attention over the mixed cache, with no
 *     separate refresh pass.
 *
 * Exactly cs_kv_refresh_scatter(k_new, v_new, slot, ..., n_tok, ...) followed by
 * cs_window_prefill_attn(q, ..., plan_mode, ...) on the same layer, same arguments, same results
 * bit for bit.  CS_BF16 with head_dim 128: ONE launch: every workgroup of the persistent attention
 * grid first moves its share of the new rows (stores written through to memory at device scope),
 * the grid meets at a launch-wide barrier, then attention proceeds as in cs_window_prefill_attn; a
 * CS_ATTN_PLAN_BUILD call is preceded by the planning launch, a CS_ATTN_PLAN_ONLY call plans and
 * moves nothing.  Other shapes: the two calls are queued one after the other.
 *
 * The barrier needs the whole grid (at most 512 workgroups, two per CU) resident at once, which a
 * device with all 256 CUs free for the launch gives.  Its wait is bounded so that every wave exits;
 * if it ever expires (part of the grid could not become resident) the 32-bit word at byte offset
 * CS_ATTN_STATUS_OFFSET of the workspace is 1 after the call has completed and the call's results
 * are not valid; it is 0 otherwise (the planning launch clears it, together with the barrier's
 * counters: after a call that raised the word, plan again with CS_ATTN_PLAN_BUILD before the
 * workspace serves another call).
 *
 * Measured on MI355X as eager calls the one launch is 17 % shorter than the two calls for a single
 * stream (26 against 32 us) and within 3 % of them for batches of 32-64 streams (there the row move
 * is bandwidth-bound, so the launch saved is about what the barrier adds); replayed from a HIP
 * graph, where a kernel boundary costs about 2 us, the step built on it is 3-12 % longer than the
 * step of separate calls.
 *
 *  k_new, v_new, slot, n_tok    as in cs_kv_refresh_scatter (slot < 0 skips the row)
 *  k_cache_layer, v_cache_layer i/o
 *  all other arguments          as in cs_window_prefill_attn
 * Errors: those of the two calls; the attention call's arguments are checked before anything is
 * queued, so a call that returns an argument error has moved no row.
 * ------------------------------------------------------------------------------------------ */
#define CS_ATTN_STATUS_OFFSET 56   /* byte offset of the barrier status word in the attention workspace */

int cs_refresh_prefill_attn(const void* k_new, const void* v_new, const int32_t* slot, int64_t n_tok,
                            const void* q, void* k_cache_layer, void* v_cache_layer,
                            const int32_t* cu_q, const int32_t* q_pos, const int32_t* kv_len,
                            const int32_t* block_table, int32_t max_blocks, int32_t block_size,
                            void* out, int64_t n_q, int32_t n_streams,
                            int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                            int64_t stride_slot, int64_t stride_head, float softmax_scale,
                            int32_t dtype, void* workspace, size_t workspace_bytes,
                            int32_t plan_mode, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CODECSIGHT_H_ */
