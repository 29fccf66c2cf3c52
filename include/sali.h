/*
 * sali.h - C ABI of the Sali-Cache pre-attention filter for AMD MI355X (gfx950).
 *
 * The library implements the per-frame work the method does before any attention
 * (Methodology; Algorithm 1):
 *   - temporal filter: dense optical flow between consecutive frames, per-patch motion
 *     (Eq. 5), frame redundancy score (Eq. 6) and the reuse rule R_frame > theta_R;
 *   - spatial filter: Canny + LAB colour-variance saliency map pooled per patch (Eq. 7)
 *     and the four storage tiers FP16 / INT8 / INT4 / Prune (Eq. 8);
 *   - storing each new frame's K/V rows at the precision of their tier (Algorithm 1,
 *     "Store (K_i, V_i) with precision Q(s_i)"; Implementation Details: symmetric min-max
 *     INT8, asymmetric INT4) in compacted pools, and expanding them again on read
 *     (Just-In-Time Dequantization).
 *   - attention of one layer over the compressed cache with the dequantisation fused in
 *     (Implementation Details), for one query per head up to 64 queries per K/V head.
 *
 * Conventions
 *   - Every pointer named d_* is DEVICE memory owned by the caller.  The library never
 *     allocates or frees device memory; it launches kernels on the HIP stream passed as
 *     `void* stream` (a hipStream_t, NULL = the default stream) and returns at once.
 *     Buffers must stay alive and unmodified until the stream has passed that point.
 *   - Pointers named h_* are HOST memory.
 *   - Calls return SALI_OK (0) or a negative SALI_ERR_* for argument errors found on the
 *     host; nothing is launched in that case.  Conditions only the device can see (pool
 *     overflow, non-finite input) set sticky bits in a device status word read by
 *     sali_get_status.
 *   - Calls on one context must be issued from one host thread at a time and on one
 *     stream (or on streams the caller orders); the context keeps the previous frame's
 *     polynomial expansion and the pool cursors between calls.
 *   - Token i of a frame is patch (row r, column c) of the grid x grid partition,
 *     i = grid * r + c; patch r covers source rows [floor(r*H/grid), floor((r+1)*H/grid)).
 */
#ifndef SALI_H
#define SALI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SALI_OK             0
#define SALI_ERR_NULL      -1   /* a required pointer is NULL                                */
#define SALI_ERR_SHAPE     -2   /* frame id / count / size outside the configured range      */
#define SALI_ERR_ALIGN     -3   /* K/V or workspace pointer not 16-byte (256 for workspaces) aligned */
#define SALI_ERR_CONFIG    -4   /* inconsistent sali_config                                  */
#define SALI_ERR_STATE     -5   /* call not valid in the context's current state             */
#define SALI_ERR_HIP       -6   /* the HIP runtime reported an error on launch / copy        */

/* sticky device status bits (sali_get_status) */
#define SALI_FAULT_OVERFLOW    0x1u   /* a pool had no room: that frame was recorded as not stored */
#define SALI_FAULT_NONFINITE   0x2u   /* an inf/NaN K/V value was met while storing                */
#define SALI_FAULT_NAN_SCORE   0x4u   /* a NaN saliency score: that frame was recorded as not stored */
#define SALI_FAULT_NO_DATA     0x8u   /* sali_kv_decompress of a frame that holds no data          */

/* tier codes (Eq. 8) */
#define SALI_TIER_FP16  0
#define SALI_TIER_INT8  1
#define SALI_TIER_INT4  2
#define SALI_TIER_PRUNE 3

#define SALI_TOKENS_MAX 576     /* grid * grid; grid is 24 (576 visual tokens per frame)     */
#define SALI_MAX_BATCH 16       /* frames that one sali_analyze_batch call may take               */
#define SALI_ANALYSIS_LANES 32  /* frames whose image-side analysis may be in flight at once      */

typedef struct sali_ctx sali_ctx;   /* opaque host object; owns no device memory */

typedef struct sali_config {
    int32_t src_h, src_w;            /* source frame size in pixels, each >= grid                      */
    int32_t grid;                    /* patches per side; must be 24                                   */
    int32_t flow_levels;             /* pyramid levels (scale 0.5), 1..6; the paper uses 3             */
    int32_t flow_iters;              /* displacement updates per level, 1..8 (3)                       */
    float   tau_t;                   /* Eq. 5/6: patch i is static iff Delta P_i < tau_t (pixels)      */
    float   theta_r;                 /* frame is redundant iff R_frame > theta_r                       */
    int32_t canny_lo, canny_hi;      /* Sobel-magnitude thresholds, 1 <= lo <= hi <= 1442              */
    int32_t tier_mode;               /* 0: thresholds of Eq. 8; 1: top-k counts; 2: Eq. 8 with adaptive
                                        thresholds (see "Adaptive thresholds" below)                   */
    float   tau_high, tau_med, tau_low;      /* mode 0, tau_low <= tau_med <= tau_high                 */
    int32_t k_fp16, k_int8, k_int4;  /* mode 1: tokens per tier by descending score; rest pruned;
                                        mode 2: the target counts the thresholds are steered to        */
    int32_t n_layers, n_heads;       /* K/V shape [n_layers][2][n_heads][576][head_dim]                */
    int32_t head_dim;                /* must be 128                                                    */
    int32_t group;                   /* quantisation group along head_dim; must be 32                  */
    int64_t cap_fp16, cap_int8, cap_int4;    /* pool capacities in tokens (rows per layer/K|V/head),
                                                each below 2^24                                          */
    int32_t max_frames;              /* frame ids are 0 .. max_frames-1                                */
    int32_t budget_tokens;           /* memory budget in cached patches (Experimental Setup: 784); 0 = none,
                                        else >= 576.  See "Memory budget" below.                        */
    int32_t tiles_per_frame;         /* images of 576 patches that make up one video frame, 1..8; 0 reads as 1.
                                        See "Dynamic-resolution frames" below.                          */
    int32_t adapt_rate_q8;           /* mode 2: step of the threshold update in 1/256, 0..256          */
} sali_config;

/* Memory budget (Experimental Setup: the methods are compared under a strict budget of 784 patches; the
 * paper states no eviction rule for its own cache, this is the library's).  With budget_tokens > 0 the
 * cache holds at most that many patches (tokens kept at any precision; pruned tokens and pointer entries
 * hold nothing).  When a frame is about to be stored, the oldest stored frames are evicted whole, oldest
 * first, until the new frame's kept tokens fit the budget and its rows fit the pools, which are rings in
 * this mode: a frame's rows of one pool stay one run [base, base + n), placed at the pool's cursor if the
 * run ends inside the pool, else at row 0, and never on rows of a frame still held.  An evicted frame and
 * every pointer entry that referred to it hold no data afterwards: their rows read src = -1, stored = 0,
 * sali_kv_decompress returns zeros and sets SALI_FAULT_NO_DATA, attention skips them.  A frame that an
 * empty cache cannot hold (a pool smaller than its rows) is recorded as not stored (SALI_FAULT_OVERFLOW).
 * Frame ids must increase from call to call (SALI_ERR_STATE otherwise).  Eviction happens when a frame is
 * analysed (sali_analyze*, sali_step*, sali_kv_compress), so reads of a frame issued after a later
 * frame's analysis may already find it evicted; within one batch the frames are taken in order, and a
 * frame evicted by a later frame of its own batch is never written. */

/* Adaptive thresholds (the Discussion says the thresholds need tuning per video domain, the Conclusion
 * names adaptive thresholds as future work; the paper gives no rule, this is the library's).  With
 * tier_mode = 2 every stored frame is tiered by Eq. 8 with the thresholds in force, and afterwards each
 * threshold moves adapt_rate_q8 / 256 of the way to the score quantile that would have given its tier the
 * target count in that frame: q_high = the score of rank k_fp16 in (score descending, token index
 * ascending) order, q_med at rank k_fp16 + k_int8, q_low at rank k_fp16 + k_int8 + k_int4 (0 if there is no
 * such rank).  Thresholds and quantiles are integers in units of 2^-16 (floor; the scores of
 * sali_saliency_pool are exact multiples): tau <- tau + floor((q - tau) * adapt_rate_q8 / 256).  The state
 * lives in device memory, starts at sali_create / sali_reset from tau_high, tau_med, tau_low, is carried from
 * stored frame to stored frame in video order (pointer frames and frames that could not be stored leave it
 * alone) and is what sali_kv_compress uses too.  adapt_rate_q8 = 0 is Eq. 8 with fixed thresholds. */

/* Dynamic-resolution frames (Background, Adapter Projection: the vision encoder of the model the paper
 * uses cuts a high-resolution frame into several images of 576 patches each, so a frame has a multiple of
 * 576 visual tokens).  With tiles_per_frame = T > 1 a video frame is T images ("tiles") of src_h x src_w
 * pixels; its N_p = 576 T patches are the patches of all of them.  Every tile is a cache entry of its own:
 * entry id e = t T + j for tile j of frame t, and wherever this header says "frame id", "frame-table row"
 * or "frames" of a batch, entries are meant (max_frames counts entries; the K/V of an entry is
 * [n_layers][2][n_heads][576][head_dim]).  The analysis calls take whole video frames: first id and count
 * multiples of T (SALI_ERR_SHAPE otherwise; so sali_step / sali_analyze need T = 1, tiled frames go through
 * the batched calls, up to SALI_MAX_BATCH / T frames per call).  The flow of a tile is taken against the
 * same tile of the adjacent frame; Eq. 6 counts the static patches of all T tiles, and the reuse rule takes
 * one decision for the frame (sali_gate then holds the frame's n_static out of 576 T in every entry); the
 * entries of a redundant frame point at the last stored entry of their own tile; otherwise each tile gets
 * its saliency scores and tiers (Eq. 8 per patch; the top-k counts apply per tile) and is stored.
 * Not combined with a memory budget (SALI_ERR_CONFIG). */

/* Result of the temporal filter for one frame pair (Eq. 6 and the reuse rule). */
typedef struct sali_gate {
    int32_t n_static;                /* #{i : Delta P_i < tau_t}                                       */
    float   r_frame;                 /* n_static / 576                                                 */
    int32_t redundant;               /* r_frame > theta_r                                              */
    int32_t reserved;
} sali_gate;

/* One frame-table row (Algorithm 1: C[t] is either stored data or a pointer). */
typedef struct sali_frame_row {
    int32_t frame_id;
    int32_t src;                     /* frame whose pool rows hold this frame's K/V; -1 = none         */
    int32_t stored;                  /* 1: this frame wrote pool rows; 0: pointer or failed            */
    int32_t base16, base8, base4;    /* first pool row (per plane) of this frame in each pool          */
    int32_t n16, n8, n4, n_pruned;   /* tokens per tier; sum = 576 when stored                         */
    int32_t reserved[2];
} sali_frame_row;

/* Byte offsets of the six arrays inside the caller's pool buffer: fp16 rows (head_dim halves),
 * int8 codes (head_dim bytes), int8 scales (head_dim/32 fp32), int4 codes (head_dim/2 bytes,
 * element 2j in the low nibble of byte j), int4 scales (fp32), int4 zero-points (fp16).
 * Each array holds cap * P rows, P = n_layers * 2 * n_heads planes (plane = (layer * 2 + K|V) *
 * n_heads + head), laid out frame by frame: a stored frame whose frame-table row says base = b and
 * n rows for that pool owns rows [b * P, (b + n) * P) of the array, and plane p of the frame owns
 * rows [b * P + p * n, b * P + (p + 1) * n) in compaction order.  So all a frame writes to one
 * array is a single contiguous range. */
typedef struct sali_pool_layout {
    uint64_t off_fp16, off_codes8, off_scale8, off_codes4, off_scale4, off_zero4;
    uint64_t total_bytes;
} sali_pool_layout;

/* Sizes of the three device buffers sali_create needs for `cfg`.  Host only. */
int sali_workspace_bytes(const sali_config* cfg, size_t* scratch_bytes, size_t* pool_bytes,
                         size_t* table_bytes);

/* Where each pool array lies inside the pool buffer.  Host only. */
int sali_pool_offsets(const sali_config* cfg, sali_pool_layout* out);

/* Build a context over three caller-owned device buffers (256-byte aligned, at least the
 * sizes sali_workspace_bytes reports).  Synchronous: clears the tables and uploads the
 * colour look-up tables with blocking copies on the current device.  The pools are not
 * cleared.  On error *out is NULL. */
int sali_create(const sali_config* cfg, void* d_scratch, void* d_pools, void* d_tables,
                sali_ctx** out);

/* Frees the host object only; pending work on the caller's stream is the caller's to wait for. */
void sali_destroy(sali_ctx* ctx);

/* Forget all frames: cursors, frame table, status word and the cached previous frame.
 * Asynchronous on `stream`. */
int sali_reset(sali_ctx* ctx, void* stream);

/* Change the temporal thresholds (Eq. 5/6; Discussion: thresholds may need tuning per
 * video domain).  Applies to calls issued afterwards. */
int sali_set_gate_thresholds(sali_ctx* ctx, float tau_t, float theta_r);

/* Change the spatial thresholds or the top-k counts that turn scores into tiers (Eq. 8), for callers
 * that steer them themselves (tier_mode 2 is the built-in policy).  tier_mode, thresholds and
 * counts as in sali_config, same consistency rules (SALI_ERR_CONFIG otherwise, nothing changes); in
 * mode 2 the thresholds in force are not touched (they restart from the configuration at sali_reset).
 * Applies to frames analysed or compressed by calls issued afterwards; frames already in the
 * cache keep their tiers. */
int sali_set_tier_params(sali_ctx* ctx, int32_t tier_mode, float tau_high, float tau_med, float tau_low,
                         int32_t k_fp16, int32_t k_int8, int32_t k_int4);

/* Temporal filter on an explicit frame pair (Temporal Filtering via Optical Flow; Eq. 5,
 * Eq. 6): dense flow from d_prev_rgb to d_cur_rgb (uint8 [H][W][3]), then
 *   d_patch_motion576[i] = sqrt(mean over patch i of u^2 + v^2)        (fp32, 576 values)
 *   *d_gate_out          = {n_static, r_frame, redundant}               (sali_gate, device)
 * d_flow_uv_or_null, if given, receives the flow as fp32 [2][H][W] (u plane, then v plane);
 * flow (u, v) at (x, y) means the content at (x, y) of prev appears at (x+u, y+v) in cur.
 * Does not touch the frame history used by sali_step. */
int sali_flow_score(sali_ctx* ctx, const uint8_t* d_prev_rgb, const uint8_t* d_cur_rgb,
                    float* d_flow_uv_or_null, float* d_patch_motion576, sali_gate* d_gate_out,
                    void* stream);

/* Spatial filter (Spatial Filtering via Saliency-Guided Quantization; Eq. 7): saliency map
 * of d_rgb (uint8 [H][W][3]) pooled per patch.
 *   d_scores576[i]     = floor(q_i * 2^15 / |P_i|) / 65536, q_i = sum over patch i of (E + C)
 *   d_salmap_or_null   = E + C in {0, 1, 2} per pixel, uint8 [H][W]  (the map S is half of it) */
int sali_saliency_pool(sali_ctx* ctx, const uint8_t* d_rgb, uint8_t* d_salmap_or_null,
                       float* d_scores576, void* stream);

/* Tier assignment (Eq. 8, or top-k counts in mode 1), compaction and storage of one frame
 * (Algorithm 1, "Store (K_i, V_i) with precision Q(s_i)").
 *   d_kv_fp16   : fp16 [n_layers][2][n_heads][576][head_dim], 16-byte aligned; index 0 of
 *                 the second axis is K, 1 is V
 *   d_scores576 : fp32 saliency per token, from sali_saliency_pool or any other source
 *   frame_id    : row of the frame table to fill, 0 <= frame_id < max_frames
 * Pool rows are appended at the cursors; if any pool lacks room the frame is recorded as
 * not stored and SALI_FAULT_OVERFLOW is set. */
int sali_kv_compress(sali_ctx* ctx, const void* d_kv_fp16, const float* d_scores576,
                     int32_t frame_id, void* stream);

/* Dequantise-on-read (Just-In-Time Dequantization): rebuild frame `frame_id` (or the frame
 * its pointer refers to) as dense fp16 [n_layers][2][n_heads][576][head_dim] in token order.
 * FP16-tier rows are bit-identical to what was stored, pruned rows are zeros.
 * d_valid576_or_null, if given, receives 1 for kept tokens and 0 for pruned ones. */
int sali_kv_decompress(sali_ctx* ctx, int32_t frame_id, void* d_kv_fp16_out,
                       uint8_t* d_valid576_or_null, void* stream);

/* One loop body of Algorithm 1 for frame `frame_id` with image d_rgb_t and K/V d_kv_t:
 * flow against the frame of the previous sali_step call (the adjacent frame, whether or not it
 * was stored) -> gate; a redundant frame becomes a pointer row to the last stored frame: no
 * ranking, no tiers, no K/V read or written; otherwise saliency -> tiers -> storage as in
 * sali_kv_compress.  The first call after create/reset has no previous frame and always
 * stores.  No host synchronisation: the gate lives in device memory and later kernels
 * test it: the temporal filter runs first (gray, pyramid, expansion, flow, per-patch motion), and the
 * kernels of the spatial filter go by the reuse rule evaluated from the motions and leave at once for
 * a redundant frame, so such a frame costs its temporal filter and nothing else (Algorithm 1). */
int sali_step(sali_ctx* ctx, const uint8_t* d_rgb_t, const void* d_kv_t, int32_t frame_id,
              void* stream);

/* The two halves of sali_step, for callers that overlap them.  The decision of Algorithm 1
 * needs only the image, and a redundant frame needs no K/V at all, so the image side of later
 * frames can run while the K/V of frame t is still being stored.
 *
 * sali_analyze: temporal filter against the previously analysed frame, and for a non-redundant
 * frame saliency, tiers and compaction indices; fills the frame-table row of `frame_id`
 * (pointer row if redundant).  Asynchronous on `stream`.  Frames must be analysed in video
 * order.  Consecutive calls may use different streams: the context keeps SALI_ANALYSIS_LANES
 * copies of its image scratch, so that many analyses can be in flight, and orders what must
 * be ordered (a frame's flow after its predecessor's expansion, tier assignment in frame
 * order, reuse of a scratch copy after its previous user) with device-side event waits.
 * sali_flow_score and sali_saliency_pool share one of the scratch copies: do not run them
 * while analyses are in flight on other streams.
 *
 * sali_store: packs `d_kv_fp16` into the pools according to the row that sali_analyze wrote.
 * Makes `stream` wait (on the device) for that frame's analysis if it ran on another stream.
 * SALI_ERR_STATE if `frame_id` is not among the last 2 * SALI_ANALYSIS_LANES analysed frames.
 *
 * sali_step(ctx, rgb, kv, id, s) == sali_analyze(ctx, rgb, id, s); sali_store(ctx, kv, id, s).
 *
 * sali_analyze_batch: the analysis of `n_frames` (1..SALI_MAX_BATCH) consecutive frames with ids
 * first_frame_id, first_frame_id + 1, ... in ONE set of kernel launches (the frame is a grid
 * dimension).  `d_rgb_frames` is a HOST array of n_frames device pointers, read before the call
 * returns; the images must stay unchanged until the work on `stream` has run.  Results are
 * identical to n_frames calls of sali_analyze: a frame's flow is taken against the frame before
 * it (the last frame of the previous call for the first of the batch) and tiers and pool rows
 * are handed out in frame order.  One 336x336 frame cannot fill 256 compute units and every
 * kernel boundary disturbs a bandwidth-bound kernel on another stream, so batches are both
 * faster and quieter.  SALI_ERR_SHAPE if n_frames or the ids are out of range. */
int sali_analyze(sali_ctx* ctx, const uint8_t* d_rgb, int32_t frame_id, void* stream);
int sali_analyze_batch(sali_ctx* ctx, const uint8_t* const* d_rgb_frames, int32_t first_frame_id, int32_t n_frames,
                       void* stream);
int sali_store(sali_ctx* ctx, const void* d_kv_fp16, int32_t frame_id, void* stream);

/* The K/V side in batches, for the same two reasons.  Frame i of a call has id first_frame_id + i;
 * the pointer arrays are HOST arrays of n_frames (1..SALI_MAX_BATCH) device pointers (each K/V
 * buffer dense fp16 [n_layers][2][n_heads][576][128], 16-byte aligned), read before the call
 * returns.  One launch each; results identical to n_frames single calls.
 *   sali_store_batch          packs the frames according to their rows (all must have been analysed)
 *   sali_kv_decompress_batch  dequantise-on-read of n_frames frames; d_valid_or_null, if given,
 *                             receives n_frames * 576 bytes (1 = token present)
 *   sali_step_batch           sali_analyze_batch followed by sali_store_batch on one stream */
int sali_store_batch(sali_ctx* ctx, const void* const* d_kv_frames, int32_t first_frame_id, int32_t n_frames,
                     void* stream);
int sali_kv_decompress_batch(sali_ctx* ctx, int32_t first_frame_id, int32_t n_frames,
                             void* const* d_kv_fp16_out_frames, uint8_t* d_valid_or_null, void* stream);
int sali_step_batch(sali_ctx* ctx, const uint8_t* const* d_rgb_frames, const void* const* d_kv_frames,
                    int32_t first_frame_id, int32_t n_frames, void* stream);

/* Just-In-Time Dequantization, fused with attention (Implementation Details): single-query
 * attention of one layer over the cache, reading the mixed-precision pools directly.  For every
 * head h:  s_j = softmax_scale * <q_h, K^_j>,  out_h = sum_j softmax(s)_j V^_j,
 * lse_h = log sum_j exp(s_j), over the logical token sequence of frames frame_lo .. frame_hi - 1:
 * every frame contributes the kept tokens of its cache entry, a redundant frame (pointer entry)
 * those of its source frame once more, pruned tokens and frames without data nothing.  "Fused" is
 * taken literally: K^, V^ are the stored codes times their fp32 scales (plus the fp16 zero-point
 * for INT4) as exact real numbers, evaluated in fp32 and never rounded to fp16 on the way; FP16 rows
 * as stored.  (sali_kv_decompress rounds the same numbers to fp16, so attention over its output
 * differs from this call by up to 2^-11 relative per K^ / V^ element.)  With lse the caller can merge
 * the result with attention over other keys (text tokens).
 *   d_q_fp16   device, fp16 [n_heads][128], 16-byte aligned
 *   d_out      device, fp32 [n_heads][128]; zeros where the range holds no token
 *   d_lse_or_null  device, fp32 [n_heads]; -inf where the range holds no token
 * Asynchronous on `stream`, which must be ordered after the stores of the frames read.  Uses one
 * partial-result area of the context: calls on one context must not overlap each other.
 * SALI_ERR_SHAPE if layer or the frame range is out of range (frame_lo == frame_hi is allowed). */
int sali_attend_decode(sali_ctx* ctx, int32_t layer, const void* d_q_fp16, int32_t frame_lo, int32_t frame_hi,
                       float softmax_scale, float* d_out, float* d_lse_or_null, void* stream);

/* The same with several queries per K/V head: the cache holds n_heads K/V heads (the context's
 * n_heads) and q_per_kv queries share each of them; query j reads K/V head j / q_per_kv.
 * d_q_fp16 is [n_heads * q_per_kv][128], d_out [n_heads * q_per_kv][128], d_lse_or_null
 * [n_heads * q_per_kv].  Every compressed row is still read once per call.
 *   q_per_kv in {1, 2, 4, 8}: grouped-query decode, the streaming kernel of sali_attend_decode
 *                (K^, V^ never rounded to fp16).
 *   q_per_kv in 9 .. 64:      many queries against the cache (the tokens of a prompt, or of several
 *                query heads, laid out per K/V head); the two products run on the matrix cores,
 *                whose operands are fp16: here, and only here, K^, V^ are rounded to fp16 (the
 *                values sali_kv_decompress returns) and so are the softmax weights; accumulation
 *                is fp32.
 * SALI_ERR_SHAPE for another q_per_kv. */
int sali_attend_decode_gqa(sali_ctx* ctx, int32_t layer, const void* d_q_fp16, int32_t q_per_kv, int32_t frame_lo,
                           int32_t frame_hi, float softmax_scale, float* d_out, float* d_lse_or_null, void* stream);

/* For callers that cannot allocate device memory or pass a workspace for this call (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): sali_attend_decode with its
 * partial softmax states kept in a device array that is part of the library image instead of the
 * context's scratch buffer.  Arguments, results and tolerances are those of sali_attend_decode.
 * The call allocates nothing (no hipMalloc / hipFree, no allocating library routine).
 *   - limit: the context's n_heads <= SALI_STATIC_ATTEND_MAX_HEADS, else SALI_ERR_SHAPE; the array is
 *     SALI_STATIC_ATTEND_MAX_HEADS * 256 partials * 640 B = 10 MiB on every GPU the library is used on,
 *     held until the process ends.
 *   - the array's device address is looked up once per GPU in sali_create; SALI_ERR_STATE if the
 *     current device is not the one the context was created on.
 *   - all calls on one GPU share the array (whatever the context): calls that overlap on one GPU,
 *     on different streams or contexts, race.  Nothing of a previous call's contents is read: every
 *     partial the merge step reads is written by the same call first.
 * It does not replace or share state with sali_attend_decode, which may run next to it. */
#define SALI_STATIC_ATTEND_MAX_HEADS 64
int sali_attend_decode_static(sali_ctx* ctx, int32_t layer, const void* d_q_fp16, int32_t frame_lo, int32_t frame_hi,
                              float softmax_scale, float* d_out, float* d_lse_or_null, void* stream);

/* One loop body of Algorithm 1 with look-ahead on caller-owned streams: analyses a later
 * frame `next_frame_id` (image d_rgb_next, may be NULL at the end of a sequence) on
 * `image_stream` and stores the K/V of the already analysed frame `frame_id` (d_kv, may be NULL
 * while the look-ahead fills) on `kv_stream`.  With a look-ahead of k frames the caller cycles
 * through k image streams (k <= SALI_ANALYSIS_LANES is useful).  Results are identical to
 * calling sali_step frame by frame. */
int sali_step_pipelined(sali_ctx* ctx, const uint8_t* d_rgb_next_or_null, int32_t next_frame_id,
                        const void* d_kv_or_null, int32_t frame_id, void* image_stream, void* kv_stream);

/* Copy `count` frame-table rows starting at `first` to host memory.  Waits for `stream`. */
int sali_read_frame_table(sali_ctx* ctx, sali_frame_row* h_rows, int32_t first, int32_t count,
                          void* stream);

/* Copy the tier (uint8[576]) and slot (uint16[576]) tables of a stored frame to host memory.
 * Waits for `stream`. */
int sali_read_frame_tiers(sali_ctx* ctx, int32_t frame_id, uint8_t* h_tier576, uint16_t* h_slot576,
                          void* stream);

/* Results that the most recently analysed frame (the last one of a batch) left in device
 * memory, copied to host: per-patch motion (fp32[576]), the gate, and the saliency scores
 * (fp32[576]; not computed for a redundant frame, whose 576 values are then unspecified); any
 * pointer may be NULL.  Motion and gate are zeros if the frame had no predecessor.  Waits for `stream`, which must be the stream
 * of that analysis (or ordered after it). */
int sali_read_last_step(sali_ctx* ctx, float* h_patch_motion576, sali_gate* h_gate,
                        float* h_scores576, void* stream);

/* The same for any of the SALI_ANALYSIS_LANES most recently analysed frames (each analysis keeps
 * its per-patch motion, gate and scores in its own scratch copy until that copy's next user, the
 * analysis SALI_ANALYSIS_LANES frames later, is issued): Eq. 5 motion, Eq. 6 gate and Eq. 7 scores
 * of frame `frame_id`.  Makes `stream` wait for that frame's analysis, then waits for `stream`.
 * SALI_ERR_STATE if the frame is not among those frames. */
int sali_read_analysis(sali_ctx* ctx, int32_t frame_id, float* h_patch_motion576, sali_gate* h_gate,
                       float* h_scores576, void* stream);

/* Measurement hook.  Arms one pair of caller-created HIP events (hipEvent_t, passed as void*):
 * the next launch of the chosen kernel records `start` just before and `stop` just after it on
 * the call's stream, then the pair is disarmed.  which: SALI_PROF_PACK = the storage kernel of
 * sali_step / sali_store[_batch] / sali_kv_compress, SALI_PROF_UNPACK = the kernel of
 * sali_kv_decompress[_batch] (one launch per call, whatever the batch size), SALI_PROF_ATTEND =
 * the main kernel of sali_attend_decode.  NULL
 * events disarm.  The caller reads the elapsed time after synchronising. */
#define SALI_PROF_PACK   0
#define SALI_PROF_UNPACK 1
#define SALI_PROF_ATTEND 2   /* the main kernel of sali_attend_decode */
int sali_set_profile_events(sali_ctx* ctx, int which, void* start_event, void* stop_event);

/* Read and keep the sticky device status word.  Waits for `stream`. */
int sali_get_status(sali_ctx* ctx, uint32_t* h_flags, void* stream);

/* Static text for a return code. */
const char* sali_error_string(int code);

#ifdef __cplusplus
}
#endif
#endif /* SALI_H */
