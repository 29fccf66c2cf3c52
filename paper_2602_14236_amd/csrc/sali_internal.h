// Internal declarations shared by the host API and the kernel files of libsali.
// gfx950 only; wave size 64.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "sali.h"

namespace sali {

constexpr int kGrid = 24;
constexpr int kTokens = kGrid * kGrid;      // 576 visual tokens per frame
constexpr int kHeadDim = 128;
constexpr int kGroup = 32;                  // quantisation group along head_dim
constexpr int kGroupsPerRow = kHeadDim / kGroup;
constexpr int kMaxLevels = 6;
constexpr int kMaxIters = 8;
constexpr int kAttnPartials = 256;          // partial softmax states per head in the attention kernel
constexpr int kAttnMaxQPerKv = 8;           // query heads that may share one K/V head
constexpr int kAttnSlotsPerHead = 4096;     // partial-result slots of the scratch per K/V head (shared out over its queries)
constexpr int kAttnPartialStride = 160;     // floats per partial: max, sum, 128 values; 640 B = five whole 128-byte lines
constexpr int kMaxBatch = SALI_MAX_BATCH;   // frames analysed by one set of launches (blockIdx.z / .y)
constexpr int kMaxTiles = 8;                // images per video frame (a frame's tiles are analysed in one batch)

// flow constants (polynomial expansion 7x7 sigma 1.5; aggregation window 11x11 sigma 2.5;
// prior-centred ridge term lambda = kLamAbs + kLamRel * trace(G) / 2)
constexpr int kPolyN = 3;
constexpr float kPolySigma = 1.5f;
constexpr int kWinR = 5;
constexpr float kWinSigma = 2.5f;
constexpr float kLamAbs = 1e-4f;
constexpr float kLamRel = 1e-2f;

constexpr uint32_t kVMin = 10000u;          // floor of the colour-variance mask

// Device-resident bookkeeping (lives in the caller's table buffer).
// Memory-budget mode: the frames still held form a queue (oldest first) and each pool is a ring.
// The rows of the held frames of a pool are the cyclic window tail .. head (head = the pool's cursor);
// `wrapped` says that the window passes the end of the pool, in which case the rows before the wrap
// end at `end` (the cursor's value when a frame did not fit behind it and went to row 0).
struct RingState {
    int32_t oldest;             // oldest stored frame still held, -1 = none
    int32_t live_tokens;        // kept tokens of the held frames
    int32_t tail[3], end[3], live_rows[3], wrapped[3];
};

struct Cursors {
    int32_t c16, c8, c4;        // next free row of each pool
    int32_t last_src;           // frame id of the last stored frame, -1 = none
    uint32_t status;            // sticky SALI_FAULT_* bits
    uint32_t pad[3];
    RingState ring;             // used with a memory budget only
    int32_t last_src_tile[kMaxTiles];   // tiled frames: last stored entry of each tile, -1 = none
    int32_t adapt_tau[3];       // adaptive thresholds in force (tier_mode 2), units of 2^-16
    uint32_t pad2[3];
};

// The six pool arrays.  Layout of each: frame-major.  A stored frame with first row `base` and
// `n` rows in a pool owns rows [base * n_planes, (base + n) * n_planes) of the flat array, and inside
// that run plane p (layer, K|V, head) owns rows [p * n, (p + 1) * n): everything one frame writes
// to a pool is one contiguous range, whatever the capacity (with one big [plane][cap] array per
// pool a frame touched n_planes ranges megabytes apart, which cost the pack kernel 8-16 % of its
// bandwidth).
struct Pools {
    uint16_t* p16;              // fp16 bit patterns
    int8_t* c8;
    float* s8;
    uint8_t* c4;
    float* s4;
    uint16_t* z4;
    int32_t cap16, cap8, cap4;
    int32_t n_planes;
};

// first flat row of plane `plane` of a frame whose run starts at `base` and has `n` rows per plane
__host__ __device__ inline size_t pool_row0(const Pools& p, int base, int n, size_t plane) {
    return (size_t)base * (size_t)p.n_planes + plane * (size_t)n;
}

struct TierParams {
    int32_t mode;               // 0: Eq. 8 thresholds, 1: top-k counts, 2: adaptive thresholds (k = target counts)
    float tau_high, tau_med, tau_low;
    int32_t k16, k8, k4;
    int32_t adapt_q8;           // mode 2: step of the threshold update in 1/256
};

// everything the tier / compaction step needs when it is fused into another kernel; in a batched
// launch frame i of the batch has id frame_id + i and its tables follow at i * kTokens
struct TierLaunch {
    TierParams tp;
    int32_t frame_id;
    sali_frame_row* rows;
    uint8_t* tier;
    uint16_t* slot;
    uint16_t* order;
    Cursors* cur;
    int32_t cap16, cap8, cap4;
    int32_t budget;             // most tokens the cache may hold, 0 = no budget
    int32_t tiles;              // images per video frame (entries per frame), >= 1
};

struct LevelGeom {
    int32_t h[kMaxLevels];
    int32_t w[kMaxLevels];
    int64_t off[kMaxLevels];    // pixel offset of the level inside a concatenated per-level array
    int32_t tiles_x[kMaxLevels];
    int32_t tile_start[kMaxLevels + 1];   // first block index of each level in a fused launch
    int32_t levels;
};

// Per-frame operands of the batched image kernels: entry i belongs to frame i of the batch.
struct PrepBatch {
    const uint8_t* rgb[kMaxBatch];
    uint8_t* y8[kMaxBatch];
    uint8_t* cls[kMaxBatch];
    uint32_t* var[kMaxBatch];
    uint32_t* parent[kMaxBatch];
    unsigned long long* msum_acc[kMaxBatch];      // frame sum of the colour variance, accumulated
    unsigned long long* msum_clear[kMaxBatch];    // the accumulator of the lane's next use, cleared
    const float* dp[kMaxBatch];                   // the frame's per-patch motions, for the reuse rule; NULL: never redundant
    uint32_t* skip[kMaxBatch];                    // the pre-pass leaves the rule's answer here (1: redundant, no saliency)
};

// The reuse rule (Eq. 6, R_frame > theta_R) as the kernels that come after the flow evaluate it for
// themselves: tiles = images per video frame (their patches count together).
struct GateParams {
    float tau_t, theta_r;
    int32_t tiles;
};

// A polynomial expansion is stored as 20 bytes per pixel and level: Ab = {A_xx, A_xy, A_yy, b_x} and
// by = b_y (a float4 for A plus a float2 for b would be 24, a fifth of it padding, and the flow
// updates re-read both frames' expansions once per update: at 1920x1080 that is most of the image
// side's HBM traffic).
struct ExpandBatch {
    const uint8_t* y8[kMaxBatch];
    float4* A[kMaxBatch];
    float* b[kMaxBatch];
};

struct PyrBatch {                                 // per-level path (more than three levels)
    const uint8_t* y8[kMaxBatch];
    float* pyr[kMaxBatch];                        // all levels of the frame's pyramid, LevelGeom offsets
    float4* A[kMaxBatch];
    float* b[kMaxBatch];
};

struct FlowBatch {                                // expansions at level 0; the launcher adds the level offset
    const float4* A1[kMaxBatch];
    const float* b1[kMaxBatch];
    const float4* A2[kMaxBatch];
    const float* b2[kMaxBatch];
    const float2* d_in[kMaxBatch];
    float2* d_out[kMaxBatch];
};

struct PoolBatch {
    const uint8_t* cls[kMaxBatch];
    const uint32_t* parent[kMaxBatch];
    const uint32_t* var[kMaxBatch];
    const unsigned long long* msum[kMaxBatch];
    float* scores[kMaxBatch];
    const float2* flow[kMaxBatch];                // NULL: no predecessor (never redundant)
    float* dp_out[kMaxBatch];                     // per-patch motion, written by the motion launch
    const float* dp[kMaxBatch];                   // the same for the reuse rule; NULL: never redundant
    const uint32_t* skip[kMaxBatch];              // what the pre-pass found (1: redundant, no scores)
    sali_gate* gate[kMaxBatch];
    struct TierCounts* tcounts[kMaxBatch];        // hand-over from the frame's ranking to the row writer
};

struct KvBatch {
    void* kv[kMaxBatch];
};

struct FlowWeights {
    float poly_g[2 * kPolyN + 1];    // normalised Gaussian of the expansion
    float win_g[2 * kWinR + 1];      // normalised Gaussian of the aggregation window
    float inv_m2;                    // 1 / m2
    float inv_den;                   // 1 / (m4 - m2^2)
    float inv_2m2sq;                 // 1 / (2 m2^2)
    float m2;
};

// XCD-aware block order.  The hardware deals the workgroups of a launch round-robin to the 8 XCDs
// in linear-id order (x fastest), and every XCD has an L2 of its own: with the plain order
// neighbouring tiles land on different XCDs and every L2 ends up holding every frame.  This maps
// the hardware id to a logical (x, y, z) such that each XCD works through one contiguous run of the
// (z, y, x) order: tiles that share halos share an L2, and an L2 holds an eighth of the data.
struct BlockId {
    int x, y, z;
};
#ifdef __HIPCC__
__device__ __forceinline__ BlockId xcd_block_id() {
    constexpr int kXcds = 8;
    const int gx = (int)gridDim.x, gy = (int)gridDim.y;
    const int total = gx * gy * (int)gridDim.z;
    const int linear = (int)blockIdx.x + gx * ((int)blockIdx.y + gy * (int)blockIdx.z);
    const int q = total / kXcds, r = total % kXcds;
    const int xcd = linear % kXcds, slot = linear / kXcds;
    const int logical = xcd * q + (xcd < r ? xcd : r) + slot;      // XCDs 0..r-1 hold q + 1 blocks
    BlockId b;
    b.z = logical / (gx * gy);
    const int rem = logical - b.z * (gx * gy);
    b.y = rem / gx;
    b.x = rem - b.y * gx;
    return b;
}
#endif

// ---- launchers (each returns hipGetLastError()) ---------------------------------------------
// kv_kernels.hip
hipError_t launch_tier(const float* d_scores, const sali_gate* d_gate_or_null, TierParams tp, int frame_id,
                       sali_frame_row* d_rows, uint8_t* d_tier, uint16_t* d_slot, uint16_t* d_order,
                       Cursors* d_cur, Pools pools, int budget, int tiles, hipStream_t s);
// frame i of a batched launch has id first_frame_id + i; f.kv[i] is its dense fp16 K/V (source of
// the pack, destination of the unpack)
hipError_t launch_pack(const KvBatch& f, int n, const sali_frame_row* d_rows, int first_frame_id,
                       const uint16_t* d_order_base, Pools pools, Cursors* d_cur, int n_planes, hipStream_t s);
hipError_t launch_unpack(const sali_frame_row* d_rows, int first_frame_id, const uint16_t* d_order_base, Pools pools,
                         const KvBatch& out, int n, uint8_t* d_valid_or_null, Cursors* d_cur, int n_planes,
                         hipStream_t s);

// attn_kernels.hip: single-query attention of one layer over frames [frame_lo, frame_hi) for
// n_heads * q_per_kv queries (q_per_kv in {1, 2, 4, 8}: streaming kernel; 9 .. 64: matrix-core kernel); d_partial holds
// n_heads * kAttnSlotsPerHead * kAttnPartialStride floats; the events (may be NULL) bracket
// the main kernel
hipError_t launch_attend(const sali_frame_row* d_rows, Pools pools, int layer, int n_heads, int q_per_kv,
                         const void* d_q, int frame_lo, int frame_hi, float softmax_scale, float* d_partial,
                         float* d_out, float* d_lse_or_null, hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t s);

// saliency_kernels.hip
// n = frames in the batch (1..kMaxBatch).  launch_gray: RGB -> gray only.  launch_prep: the edge / colour
// variance pre-pass; frames that the reuse rule finds redundant from
// f.dp are skipped (Algorithm 1: their saliency is not computed) and marked in f.skip, which launch_union
// and launch_pool go by.
hipError_t launch_gray(const PrepBatch& f, int n, int h, int w, hipStream_t s);
hipError_t launch_prep(const PrepBatch& f, int n, int h, int w, GateParams gp, const uint16_t* d_lut,
                       int lo2, int hi2, hipStream_t s);
hipError_t launch_union(const PrepBatch& f, int n, int h, int w, hipStream_t s);
// launch_motion: Eq. 5, per-patch motion of every frame of the batch from its flow (0 without flow).
// launch_pool: Eq. 7 scores (none for frames marked in f.skip);
// d_salmap_or_null applies to frame 0 (stand-alone call); with `tier` a second small launch evaluates
// the gate and assigns tiers for the n frames in order
hipError_t launch_motion(const PoolBatch& f, int n, int h, int w, hipStream_t s);
hipError_t launch_pool(const PoolBatch& f, int n, int h, int w, uint8_t* d_salmap_or_null,
                       const TierLaunch* tier_or_null, GateParams gp, uint32_t* d_done_counter, hipStream_t s);

// flow_kernels.hip
hipError_t launch_pyr_down(const PyrBatch& f, int n, const LevelGeom& g, int lvl, hipStream_t s);
hipError_t launch_polyexp(const PyrBatch& f, int n, LevelGeom g, FlowWeights fw, hipStream_t s);
hipError_t launch_expand(const ExpandBatch& f, int n, LevelGeom g, FlowWeights fw, hipStream_t s);
hipError_t launch_flow_iter(const FlowBatch& f, int n, int64_t level_off, int h, int w, int ch, int cw,
                            int prior_mode, FlowWeights fw, hipStream_t s);
hipError_t launch_patch_gate(const float2* d_flow, int h, int w, float tau_t, float theta_r, float* d_dp,
                             sali_gate* d_gate, uint32_t* d_done_counter, float* d_flow_uv_or_null, hipStream_t s);

}  // namespace sali
