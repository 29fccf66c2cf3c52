// C ABI of libsali: context management, argument checks and the per-call kernel chains.
// Every step of the method runs in the kernels of kv_kernels.hip, saliency_kernels.hip and
// flow_kernels.hip; this file only validates, lays out the caller's buffers and enqueues.

#include <math.h>
#include <mutex>
#include <new>
#include <string.h>

#include "sali_internal.h"
#include "tier_body.h"

// Partial softmax states of sali_attend_decode_static: device memory that belongs to the library
// image instead of the caller's scratch buffer, for callers that cannot allocate.  Every GPU the
// library runs on holds its own copy until the process ends.  In host code this name is only a
// stand-in for the symbol: the device address comes from hipGetSymbolAddress (static_scratch_for_device).
static __device__ __align__(256) float scratch[SALI_STATIC_ATTEND_MAX_HEADS * sali::kAttnPartials * sali::kAttnPartialStride];

namespace sali {

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Image-side scratch exists in kLanes copies (one per frame in flight) so that the analyses of
// many frames can be in flight at once, in one batch or on different streams; polynomial expansions
// live in a ring one longer than that (a frame's flow reads its predecessor's expansion), plus two
// slots for the stand-alone flow call.
constexpr int kLanes = SALI_ANALYSIS_LANES;
constexpr int kStepSlots = kLanes + 1;
constexpr int kExpSlots = kStepSlots + 2;
constexpr int kRing = 2 * kLanes;     // bookkeeping of the most recent analyses
static_assert(kLanes >= 2 * kMaxBatch, "two batches in flight");

struct LaneLayout {
    size_t y8, pyr, flow[2], cls, var, parent, msum, dp, scores, gate, counters, tcounts;
};

struct ScratchLayout {
    LaneLayout lane[kLanes];
    size_t expA[kExpSlots], expB[kExpSlots];
    size_t attn_partial;
    size_t total;
};

struct TableLayout {
    size_t lut, cursors, rows, tier, slot, order, total;      // lut = lin[256] followed by fl[4096]
};

struct LaneCounters {         // arrival counters, all self-resetting
    uint32_t patch_done;      // blocks of the stand-alone patch-motion kernel
    uint32_t skip;            // the saliency pre-pass found the lane's frame redundant (not a counter: a flag)
    uint32_t batch_done;      // frames of a pooling launch whose first frame sits in this lane
};

int check_config(const sali_config* c) {
    if (c == nullptr) return SALI_ERR_NULL;
    if (c->grid != kGrid || c->head_dim != kHeadDim || c->group != kGroup) return SALI_ERR_CONFIG;
    if (c->src_h < kGrid || c->src_w < kGrid || c->src_h > 16384 || c->src_w > 16384) return SALI_ERR_CONFIG;
    if (c->flow_levels < 1 || c->flow_levels > kMaxLevels || c->flow_iters < 1 || c->flow_iters > kMaxIters)
        return SALI_ERR_CONFIG;
    if (!(c->tau_t >= 0.0f) || !(c->theta_r >= 0.0f)) return SALI_ERR_CONFIG;
    if (c->canny_lo < 1 || c->canny_hi < c->canny_lo || c->canny_hi > 1442) return SALI_ERR_CONFIG;
    if (c->tier_mode < 0 || c->tier_mode > 2) return SALI_ERR_CONFIG;
    if (c->adapt_rate_q8 < 0 || c->adapt_rate_q8 > 256) return SALI_ERR_CONFIG;
    if (c->tier_mode != 1) {
        if (!(c->tau_low <= c->tau_med) || !(c->tau_med <= c->tau_high)) return SALI_ERR_CONFIG;
    }
    if (c->tier_mode != 0) {
        if (c->k_fp16 < 0 || c->k_int8 < 0 || c->k_int4 < 0 ||
            (long long)c->k_fp16 + c->k_int8 + c->k_int4 > kTokens)
            return SALI_ERR_CONFIG;
    }
    if (c->n_layers < 1 || c->n_heads < 1 || (long long)c->n_layers * 2 * c->n_heads > 65535) return SALI_ERR_CONFIG;
    if (c->cap_fp16 < 0 || c->cap_int8 < 0 || c->cap_int4 < 0) return SALI_ERR_CONFIG;
    // a frame's rows of one plane stay far below 4 GiB: the kernels address inside them with 32 bits
    if (c->cap_fp16 >= (1ll << 24) || c->cap_int8 >= (1ll << 24) || c->cap_int4 >= (1ll << 24)) return SALI_ERR_CONFIG;
    if (c->max_frames < 1 || c->max_frames > (1 << 24)) return SALI_ERR_CONFIG;
    // a budget holds at least one whole frame, so the newest frame can always stay
    if (c->budget_tokens != 0 && c->budget_tokens < kTokens) return SALI_ERR_CONFIG;
    if (c->tiles_per_frame < 0 || c->tiles_per_frame > kMaxTiles) return SALI_ERR_CONFIG;
    // eviction works on cache entries, a tiled frame is several: the two are not combined
    if (c->budget_tokens != 0 && c->tiles_per_frame > 1) return SALI_ERR_CONFIG;
    // the smallest pyramid level must still be an image
    int h = c->src_h, w = c->src_w;
    for (int l = 1; l < c->flow_levels; ++l) {
        h = (h + 1) / 2;
        w = (w + 1) / 2;
    }
    if (h < 2 || w < 2) return SALI_ERR_CONFIG;
    return SALI_OK;
}

LevelGeom make_geom(const sali_config& c) {
    LevelGeom g = {};
    g.levels = c.flow_levels;
    int h = c.src_h, w = c.src_w;
    int64_t off = 0;
    int tiles = 0;
    for (int l = 0; l < g.levels; ++l) {
        g.h[l] = h;
        g.w[l] = w;
        g.off[l] = off;
        g.tiles_x[l] = (w + 31) / 32;
        g.tile_start[l] = tiles;
        tiles += g.tiles_x[l] * ((h + 31) / 32);
        off += (int64_t)h * w;
        off = (off + 63) / 64 * 64;
        h = (h + 1) / 2;
        w = (w + 1) / 2;
    }
    g.tile_start[g.levels] = tiles;
    return g;
}

int64_t total_px(const LevelGeom& g) {
    return g.off[g.levels - 1] + (int64_t)g.h[g.levels - 1] * g.w[g.levels - 1];
}

FlowWeights make_weights() {
    FlowWeights fw = {};
    double pg[2 * kPolyN + 1], sum = 0;
    for (int k = -kPolyN; k <= kPolyN; ++k) {
        pg[k + kPolyN] = exp(-(double)(k * k) / (2.0 * (double)kPolySigma * (double)kPolySigma));
        sum += pg[k + kPolyN];
    }
    double m2 = 0, m4 = 0;
    for (int k = -kPolyN; k <= kPolyN; ++k) {
        pg[k + kPolyN] /= sum;
        m2 += pg[k + kPolyN] * k * k;
        m4 += pg[k + kPolyN] * k * k * k * k;
        fw.poly_g[k + kPolyN] = (float)pg[k + kPolyN];
    }
    fw.m2 = (float)m2;
    fw.inv_m2 = (float)(1.0 / m2);
    fw.inv_den = (float)(1.0 / (m4 - m2 * m2));
    fw.inv_2m2sq = (float)(1.0 / (2.0 * m2 * m2));
    double wg[2 * kWinR + 1];
    sum = 0;
    for (int k = -kWinR; k <= kWinR; ++k) {
        wg[k + kWinR] = exp(-(double)(k * k) / (2.0 * (double)kWinSigma * (double)kWinSigma));
        sum += wg[k + kWinR];
    }
    for (int k = 0; k <= 2 * kWinR; ++k) fw.win_g[k] = (float)(wg[k] / sum);
    return fw;
}

ScratchLayout scratch_layout(const sali_config& c, const LevelGeom& g) {
    ScratchLayout s = {};
    const size_t hw = (size_t)c.src_h * c.src_w;
    const size_t px = (size_t)total_px(g);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    for (int l = 0; l < kLanes; ++l) {
        LaneLayout& L = s.lane[l];
        L.y8 = take(hw);
        L.pyr = take(px * sizeof(float));
        L.flow[0] = take(hw * sizeof(float2));
        L.flow[1] = take(hw * sizeof(float2));
        L.cls = take(hw);
        L.var = take(hw * sizeof(uint32_t));
        L.parent = take(hw * sizeof(uint32_t));
        L.msum = take(2 * sizeof(unsigned long long));
        L.dp = take(kTokens * sizeof(float));
        L.scores = take(kTokens * sizeof(float));
        L.gate = take(sizeof(sali_gate));
        L.counters = take(sizeof(LaneCounters));
        L.tcounts = take(8 * sizeof(int32_t));
    }
    for (int i = 0; i < kExpSlots; ++i) {
        s.expA[i] = take(px * sizeof(float4));
        s.expB[i] = take(px * sizeof(float));
    }
    s.attn_partial = take((size_t)c.n_heads * kAttnSlotsPerHead * kAttnPartialStride * sizeof(float));
    s.total = o;
    return s;
}

TableLayout table_layout(const sali_config& c) {
    TableLayout t = {};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    t.lut = take((256 + 4096) * sizeof(uint16_t));
    t.cursors = take(sizeof(Cursors));
    t.rows = take((size_t)c.max_frames * sizeof(sali_frame_row));
    t.tier = take((size_t)c.max_frames * kTokens);
    t.slot = take((size_t)c.max_frames * kTokens * sizeof(uint16_t));
    t.order = take((size_t)c.max_frames * kTokens * sizeof(uint16_t));
    t.total = o;
    return t;
}

sali_pool_layout pool_layout(const sali_config& c) {
    sali_pool_layout p = {};
    const size_t planes = (size_t)c.n_layers * 2 * c.n_heads;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    p.off_fp16 = take(planes * (size_t)c.cap_fp16 * kHeadDim * 2);
    p.off_codes8 = take(planes * (size_t)c.cap_int8 * kHeadDim);
    p.off_scale8 = take(planes * (size_t)c.cap_int8 * kGroupsPerRow * 4);
    p.off_codes4 = take(planes * (size_t)c.cap_int4 * (kHeadDim / 2));
    p.off_scale4 = take(planes * (size_t)c.cap_int4 * kGroupsPerRow * 4);
    p.off_zero4 = take(planes * (size_t)c.cap_int4 * kGroupsPerRow * 2);
    p.total_bytes = o > 0 ? o : kAlign;
    return p;
}

struct LanePtrs {
    unsigned long long* msum;
    float* dp;
    float* scores;
    sali_gate* gate;
    LaneCounters* counters;
};

struct LanePtrArray {
    LanePtrs lane[kLanes];
};

__global__ void k_reset(Cursors* cur, sali_frame_row* rows, int max_frames, LanePtrArray lanes, int tau0, int tau1,
                        int tau2) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < max_frames) {
        sali_frame_row r = {};
        r.frame_id = -1;
        r.src = -1;
        rows[i] = r;
    }
    for (int l = 0; l < kLanes; ++l) {
        if (i < kTokens) {
            lanes.lane[l].dp[i] = 0.0f;
            lanes.lane[l].scores[i] = 0.0f;
        }
        if (i == 0) {
            lanes.lane[l].msum[0] = 0ull;
            lanes.lane[l].msum[1] = 0ull;
            sali_gate g = {0, 0.0f, 0, 0};
            *lanes.lane[l].gate = g;
            LaneCounters z = {0u, 0u, 0u};
            *lanes.lane[l].counters = z;
        }
    }
    if (i == 0) {
        Cursors c = {};
        c.last_src = -1;
        c.ring.oldest = -1;
        for (int j = 0; j < kMaxTiles; ++j) c.last_src_tile[j] = -1;
        c.adapt_tau[0] = tau0;
        c.adapt_tau[1] = tau1;
        c.adapt_tau[2] = tau2;
        *cur = c;
    }
}

}  // namespace

}  // namespace sali

using namespace sali;

// one entry of the ring of recent analyses
struct AnalysisRecord {
    int frame_id;             // -1 = empty
    hipStream_t stream;
    hipEvent_t exp_ready;     // the frame's polynomial expansion is complete
    hipEvent_t done;          // the frame's row / tier tables are complete
    int batch_last;           // ring entry whose events cover this frame (the last frame of its batch)
};

struct sali_ctx {
    sali_config cfg;
    LevelGeom geom;
    FlowWeights fw;
    ScratchLayout sl;
    TableLayout tl;
    uint8_t* scratch;
    uint8_t* tables;
    Pools pools;
    int n_planes;
    int last_frame_id;        // highest frame id handed to an analysis or to sali_kv_compress (budget mode: ids increase)
    unsigned n_analysed;      // analyses since create / reset; analysis n uses lane n % kLanes
    unsigned lane_uses[kLanes];   // saliency passes run in each lane; the parity selects the frame-sum accumulator
    AnalysisRecord ring[kRing];
    hipEvent_t prof[3][2];    // [SALI_PROF_*][start, stop], armed for one launch
    int device;               // the GPU that was current in sali_create (the buffers live there)
    float* static_scratch;    // that GPU's copy of the library's own partial-result array

    template <typename T> T* sc(size_t off) const { return reinterpret_cast<T*>(scratch + off); }
    template <typename T> T* tb(size_t off) const { return reinterpret_cast<T*>(tables + off); }
    Cursors* cursors() const { return tb<Cursors>(tl.cursors); }
    sali_frame_row* rows() const { return tb<sali_frame_row>(tl.rows); }
    uint8_t* tier(int f) const { return tb<uint8_t>(tl.tier) + (size_t)f * kTokens; }
    uint16_t* slot(int f) const { return tb<uint16_t>(tl.slot) + (size_t)f * kTokens; }
    uint16_t* order(int f) const { return tb<uint16_t>(tl.order) + (size_t)f * kTokens; }
    LanePtrs lane_ptrs(int l) const {
        const LaneLayout& L = sl.lane[l];
        LanePtrs p;
        p.msum = sc<unsigned long long>(L.msum);
        p.dp = sc<float>(L.dp);
        p.scores = sc<float>(L.scores);
        p.gate = sc<sali_gate>(L.gate);
        p.counters = sc<LaneCounters>(L.counters);
        return p;
    }
};

namespace {

#define SALI_TRY(expr)                         \
    do {                                       \
        if ((expr) != hipSuccess) return SALI_ERR_HIP; \
    } while (0)

// Which scratch copies and expansion slots the frames of one batch use.
struct BatchPlan {
    int n;                          // frames, 1..kMaxBatch
    int lane[kMaxBatch];
    int slot[kMaxBatch];            // expansion slot of the frame
    int prev_slot[kMaxBatch];       // expansion slot of its predecessor, -1 = none (first frame of a sequence)
    unsigned parity[kMaxBatch];     // which frame-sum accumulator of the lane this pass uses
};

// Pyramid and polynomial expansion in one launch (k_expand: every tile rebuilds the pyramid values it
// needs from the gray image in LDS) or level by level (k_pyr_down per level, then k_polyexp).  The fused
// launch saves two dependent launches, but does several times the work per
// pixel (a 16x16 tile of level 2 reads a 97x97 gray patch), so it is the choice only while the launch
// chain, not the work, bounds a batch: up to three levels and small frames.  Measured in the pipeline,
// eight frames per launch: 336x336 the same either way (a single frame per launch: fused 7 % faster),
// 640x360 level by level 25 100 -> 27 500 frames/s.
bool fused_expansion(const sali_ctx* c, int /*n_frames*/) {
    return c->geom.levels <= 3 && (long long)c->cfg.src_h * c->cfg.src_w < 160000;
}

GateParams gate_params(const sali_ctx* c) {
    GateParams gp;
    gp.tau_t = c->cfg.tau_t;
    gp.theta_r = c->cfg.theta_r;
    gp.tiles = c->cfg.tiles_per_frame > 1 ? c->cfg.tiles_per_frame : 1;
    return gp;
}

PrepBatch prep_batch(sali_ctx* c, const uint8_t* const* d_rgb, const BatchPlan& bp, bool with_saliency,
                     const float2* const* flow_or_null) {
    PrepBatch f = {};
    for (int i = 0; i < bp.n; ++i) {
        const LaneLayout& L = c->sl.lane[bp.lane[i]];
        unsigned long long* msum = c->sc<unsigned long long>(L.msum);
        f.rgb[i] = d_rgb[i];
        f.y8[i] = c->sc<uint8_t>(L.y8);
        f.cls[i] = c->sc<uint8_t>(L.cls);
        f.var[i] = c->sc<uint32_t>(L.var);
        f.parent[i] = c->sc<uint32_t>(L.parent);
        f.msum_acc[i] = with_saliency ? msum + (bp.parity[i] & 1u) : nullptr;
        f.msum_clear[i] = with_saliency ? msum + ((bp.parity[i] + 1u) & 1u) : nullptr;
        // a frame with a predecessor has per-patch motions by the time the pre-pass runs: the reuse rule applies
        f.dp[i] = (flow_or_null != nullptr && flow_or_null[i] != nullptr) ? c->lane_ptrs(bp.lane[i]).dp : nullptr;
        f.skip[i] = &c->lane_ptrs(bp.lane[i]).counters->skip;
    }
    return f;
}

// gray image of the batch's frames (what the flow needs)
int enqueue_gray(sali_ctx* c, const uint8_t* const* d_rgb, const BatchPlan& bp, hipStream_t s) {
    const PrepBatch f = prep_batch(c, d_rgb, bp, false, nullptr);
    SALI_TRY(launch_gray(f, bp.n, c->cfg.src_h, c->cfg.src_w, s));
    return SALI_OK;
}

// Saliency pre-pass (edges, colour variance, tile-local hysteresis) and the cross-tile hysteresis pass
// after a kernel boundary (the cheapest device-wide ordering there is).  flow_or_null: the chained step,
// after the flow and the per-patch motions: frames that the reuse rule finds redundant are skipped
// (Algorithm 1).  The other frame-sum accumulator of each lane is cleared for the lane's next use.
int enqueue_saliency(sali_ctx* c, const uint8_t* const* d_rgb, const BatchPlan& bp,
                     const float2* const* flow_or_null, hipStream_t s) {
    const sali_config& cfg = c->cfg;
    const PrepBatch f = prep_batch(c, d_rgb, bp, true, flow_or_null);
    const GateParams gp = gate_params(c);
    SALI_TRY(launch_prep(f, bp.n, cfg.src_h, cfg.src_w, gp, c->tb<uint16_t>(c->tl.lut),
                         cfg.canny_lo * cfg.canny_lo, cfg.canny_hi * cfg.canny_hi, s));
    SALI_TRY(launch_union(f, bp.n, cfg.src_h, cfg.src_w, s));
    return SALI_OK;
}

// pyramid and polynomial expansion of each frame's gray image into its expansion slot
int enqueue_expansion(sali_ctx* c, const BatchPlan& bp, hipStream_t s) {
    const LevelGeom& g = c->geom;
    if (fused_expansion(c, bp.n)) {
        ExpandBatch f = {};
        for (int i = 0; i < bp.n; ++i) {
            const LaneLayout& L = c->sl.lane[bp.lane[i]];
            f.y8[i] = c->sc<uint8_t>(L.y8);
            f.A[i] = c->sc<float4>(c->sl.expA[bp.slot[i]]);
            f.b[i] = c->sc<float>(c->sl.expB[bp.slot[i]]);
        }
        SALI_TRY(launch_expand(f, bp.n, g, c->fw, s));
        return SALI_OK;
    }
    PyrBatch f = {};
    for (int i = 0; i < bp.n; ++i) {
        const LaneLayout& L = c->sl.lane[bp.lane[i]];
        f.y8[i] = c->sc<uint8_t>(L.y8);
        f.pyr[i] = c->sc<float>(L.pyr);
        f.A[i] = c->sc<float4>(c->sl.expA[bp.slot[i]]);
        f.b[i] = c->sc<float>(c->sl.expB[bp.slot[i]]);
    }
    for (int l = 1; l < g.levels; ++l) SALI_TRY(launch_pyr_down(f, bp.n, g, l, s));
    SALI_TRY(launch_polyexp(f, bp.n, g, c->fw, s));
    return SALI_OK;
}

// coarse-to-fine displacement estimation of every frame of the batch that has a predecessor;
// flow[i] = the frame's result (NULL without predecessor)
int enqueue_flow(sali_ctx* c, const BatchPlan& bp, const float2** flow, hipStream_t s) {
    const LevelGeom& g = c->geom;
    FlowBatch f[2] = {};            // [which of the two flow buffers is read]
    int idx[kMaxBatch];
    int m = 0;
    for (int i = 0; i < bp.n; ++i) {
        flow[i] = nullptr;
        if (bp.prev_slot[i] < 0) continue;
        const LaneLayout& L = c->sl.lane[bp.lane[i]];
        for (int k = 0; k < 2; ++k) {
            f[k].A1[m] = c->sc<float4>(c->sl.expA[bp.prev_slot[i]]);
            f[k].b1[m] = c->sc<float>(c->sl.expB[bp.prev_slot[i]]);
            f[k].A2[m] = c->sc<float4>(c->sl.expA[bp.slot[i]]);
            f[k].b2[m] = c->sc<float>(c->sl.expB[bp.slot[i]]);
            f[k].d_in[m] = c->sc<float2>(L.flow[k]);
            f[k].d_out[m] = c->sc<float2>(L.flow[k ^ 1]);
        }
        idx[m++] = i;
    }
    if (m == 0) return SALI_OK;
    int cur = 0;            // buffer holding the latest estimate
    bool have = false;
    for (int l = g.levels - 1; l >= 0; --l) {
        for (int it = 0; it < c->cfg.flow_iters; ++it) {
            int mode;
            int ch = 0, cw = 0;
            if (it > 0) mode = 2;
            else if (!have) mode = 0;
            else { mode = 1; ch = g.h[l + 1]; cw = g.w[l + 1]; }
            SALI_TRY(launch_flow_iter(f[cur], m, g.off[l], g.h[l], g.w[l], ch, cw, mode, c->fw, s));
            cur ^= 1;
            have = true;
        }
    }
    for (int k = 0; k < m; ++k) flow[idx[k]] = c->sc<float2>(c->sl.lane[bp.lane[idx[k]]].flow[cur]);
    return SALI_OK;
}

PoolBatch pool_batch(sali_ctx* c, const BatchPlan& bp, float* d_scores_or_null, const float2* const* flow) {
    PoolBatch f = {};
    for (int i = 0; i < bp.n; ++i) {
        const LaneLayout& L = c->sl.lane[bp.lane[i]];
        const LanePtrs lp = c->lane_ptrs(bp.lane[i]);
        f.cls[i] = c->sc<uint8_t>(L.cls);
        f.parent[i] = c->sc<uint32_t>(L.parent);
        f.var[i] = c->sc<uint32_t>(L.var);
        f.msum[i] = lp.msum + (bp.parity[i] & 1u);
        f.scores[i] = d_scores_or_null != nullptr ? d_scores_or_null : lp.scores;
        f.flow[i] = flow != nullptr ? flow[i] : nullptr;
        f.dp_out[i] = lp.dp;
        f.dp[i] = f.flow[i] != nullptr ? lp.dp : nullptr;
        f.skip[i] = &lp.counters->skip;
        f.gate[i] = lp.gate;
        f.tcounts[i] = c->sc<TierCounts>(L.tcounts);
    }
    return f;
}

// Eq. 5: each frame's flow (NULL: no predecessor) reduced to per-patch motion
int enqueue_motion(sali_ctx* c, const BatchPlan& bp, const float2* const* flow, hipStream_t s) {
    const PoolBatch f = pool_batch(c, bp, nullptr, flow);
    SALI_TRY(launch_motion(f, bp.n, c->cfg.src_h, c->cfg.src_w, s));
    return SALI_OK;
}

// Pooling of the batch's saliency pre-pass (Eq. 7).  With `tier` (the chained step) a second launch
// evaluates the gates and writes the frame-table rows with tiers and compaction indices, in frame
// order; redundant frames get no scores.  d_scores_or_null / d_salmap redirect the outputs of a
// stand-alone single-frame call.
int enqueue_pool(sali_ctx* c, const BatchPlan& bp, float* d_scores_or_null, uint8_t* d_salmap,
                 const TierLaunch* tier, const float2* const* flow, hipStream_t s) {
    const PoolBatch f = pool_batch(c, bp, d_scores_or_null, flow);
    SALI_TRY(launch_pool(f, bp.n, c->cfg.src_h, c->cfg.src_w, d_salmap, tier, gate_params(c),
                         &c->lane_ptrs(bp.lane[0]).counters->batch_done, s));
    return SALI_OK;
}

TierParams tier_params(const sali_config& cfg) {
    TierParams tp;
    tp.mode = cfg.tier_mode;
    tp.tau_high = cfg.tau_high;
    tp.tau_med = cfg.tau_med;
    tp.tau_low = cfg.tau_low;
    tp.k16 = cfg.k_fp16;
    tp.k8 = cfg.k_int8;
    tp.k4 = cfg.k_int4;
    tp.adapt_q8 = cfg.adapt_rate_q8;
    return tp;
}

TierLaunch tier_launch(sali_ctx* c, int frame_id) {
    TierLaunch t;
    t.tp = tier_params(c->cfg);
    t.frame_id = frame_id;
    t.rows = c->rows();
    t.tier = c->tier(frame_id);
    t.slot = c->slot(frame_id);
    t.order = c->order(frame_id);
    t.cur = c->cursors();
    t.cap16 = c->pools.cap16;
    t.cap8 = c->pools.cap8;
    t.cap4 = c->pools.cap4;
    t.budget = c->cfg.budget_tokens;
    t.tiles = c->cfg.tiles_per_frame > 1 ? c->cfg.tiles_per_frame : 1;
    return t;
}

// the storage kernel of frames first_frame_id .. + n - 1; their frame-table rows and order lists
// must be in place
int enqueue_pack(sali_ctx* c, const void* const* d_kv, int first_frame_id, int n, hipStream_t s) {
    KvBatch f = {};
    for (int i = 0; i < n; ++i) f.kv[i] = const_cast<void*>(d_kv[i]);
    hipEvent_t* ev = c->prof[SALI_PROF_PACK];
    if (ev[0] != nullptr) SALI_TRY(hipEventRecord(ev[0], s));
    SALI_TRY(launch_pack(f, n, c->rows(), first_frame_id, c->tb<uint16_t>(c->tl.order), c->pools, c->cursors(),
                         c->n_planes, s));
    if (ev[1] != nullptr) SALI_TRY(hipEventRecord(ev[1], s));
    ev[0] = ev[1] = nullptr;
    return SALI_OK;
}

// make stream `s` wait for `ev` unless the event was recorded on `s` itself
int wait_unless_same(hipStream_t s, hipStream_t recorded_on, hipEvent_t ev) {
    if (recorded_on != s) SALI_TRY(hipStreamWaitEvent(s, ev, 0));
    return SALI_OK;
}

// Device address of `scratch` on the current device, looked up once per device (with that device
// current) and kept: each GPU has its own copy of the array at its own address.
constexpr int kMaxDevices = 64;
float* g_static_scratch[kMaxDevices] = {};
std::mutex g_static_scratch_lock;

int static_scratch_for_device(int* device_out, float** ptr_out) {
    int dev = -1;
    SALI_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return SALI_ERR_STATE;
    std::lock_guard<std::mutex> hold(g_static_scratch_lock);
    if (g_static_scratch[dev] == nullptr) {
        void* p = nullptr;
        SALI_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return SALI_ERR_HIP;
        g_static_scratch[dev] = static_cast<float*>(p);
    }
    *device_out = dev;
    *ptr_out = g_static_scratch[dev];
    return SALI_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

void fill_luts(uint16_t* lin, uint16_t* fl) {
    // sRGB decoding to 12-bit linear light, and the CIE L*a*b* companding function on a
    // 12-bit argument scaled by 2^15
    for (int v = 0; v < 256; ++v) {
        const double c = v / 255.0;
        const double l = c <= 0.04045 ? c / 12.92 : pow((c + 0.055) / 1.055, 2.4);
        lin[v] = (uint16_t)floor(4095.0 * l + 0.5);
    }
    const double d = 6.0 / 29.0;
    for (int t = 0; t < 4096; ++t) {
        const double u = t / 4095.0;
        const double f = u > d * d * d ? cbrt(u) : u / (3.0 * d * d) + 4.0 / 29.0;
        fl[t] = (uint16_t)floor(32768.0 * f + 0.5);
    }
}

void destroy_events(sali_ctx* c) {
    for (int i = 0; i < kRing; ++i) {
        if (c->ring[i].exp_ready != nullptr) (void)hipEventDestroy(c->ring[i].exp_ready);
        if (c->ring[i].done != nullptr) (void)hipEventDestroy(c->ring[i].done);
        c->ring[i].exp_ready = c->ring[i].done = nullptr;
    }
}

}  // namespace

extern "C" {

int sali_workspace_bytes(const sali_config* cfg, size_t* scratch_bytes, size_t* pool_bytes, size_t* table_bytes) {
    const int rc = check_config(cfg);
    if (rc != SALI_OK) return rc;
    if (scratch_bytes == nullptr || pool_bytes == nullptr || table_bytes == nullptr) return SALI_ERR_NULL;
    const LevelGeom g = make_geom(*cfg);
    *scratch_bytes = scratch_layout(*cfg, g).total;
    *pool_bytes = (size_t)pool_layout(*cfg).total_bytes;
    *table_bytes = table_layout(*cfg).total;
    return SALI_OK;
}

int sali_pool_offsets(const sali_config* cfg, sali_pool_layout* out) {
    const int rc = check_config(cfg);
    if (rc != SALI_OK) return rc;
    if (out == nullptr) return SALI_ERR_NULL;
    *out = pool_layout(*cfg);
    return SALI_OK;
}

int sali_create(const sali_config* cfg, void* d_scratch, void* d_pools, void* d_tables, sali_ctx** out) {
    if (out == nullptr) return SALI_ERR_NULL;
    *out = nullptr;
    const int rc = check_config(cfg);
    if (rc != SALI_OK) return rc;
    if (d_scratch == nullptr || d_pools == nullptr || d_tables == nullptr) return SALI_ERR_NULL;
    if (!aligned256(d_scratch) || !aligned256(d_pools) || !aligned256(d_tables)) return SALI_ERR_ALIGN;
    sali_ctx* c = new (std::nothrow) sali_ctx();
    if (c == nullptr) return SALI_ERR_STATE;
    c->cfg = *cfg;
    c->geom = make_geom(*cfg);
    c->fw = make_weights();
    c->sl = scratch_layout(*cfg, c->geom);
    c->tl = table_layout(*cfg);
    c->scratch = static_cast<uint8_t*>(d_scratch);
    c->tables = static_cast<uint8_t*>(d_tables);
    const sali_pool_layout pl = pool_layout(*cfg);
    uint8_t* pb = static_cast<uint8_t*>(d_pools);
    c->pools.p16 = reinterpret_cast<uint16_t*>(pb + pl.off_fp16);
    c->pools.c8 = reinterpret_cast<int8_t*>(pb + pl.off_codes8);
    c->pools.s8 = reinterpret_cast<float*>(pb + pl.off_scale8);
    c->pools.c4 = pb + pl.off_codes4;
    c->pools.s4 = reinterpret_cast<float*>(pb + pl.off_scale4);
    c->pools.z4 = reinterpret_cast<uint16_t*>(pb + pl.off_zero4);
    c->pools.cap16 = (int32_t)cfg->cap_fp16;
    c->pools.cap8 = (int32_t)cfg->cap_int8;
    c->pools.cap4 = (int32_t)cfg->cap_int4;
    c->n_planes = cfg->n_layers * 2 * cfg->n_heads;
    c->pools.n_planes = c->n_planes;
    c->n_analysed = 0;
    c->last_frame_id = -1;
    for (int l = 0; l < kLanes; ++l) c->lane_uses[l] = 0;
    for (int i = 0; i < 3; ++i) c->prof[i][0] = c->prof[i][1] = nullptr;
    {
        const int src = static_scratch_for_device(&c->device, &c->static_scratch);
        if (src != SALI_OK) {
            delete c;
            return src;
        }
    }
    for (int i = 0; i < kRing; ++i) {
        c->ring[i].frame_id = -1;
        c->ring[i].batch_last = i;
        c->ring[i].stream = nullptr;
        c->ring[i].exp_ready = c->ring[i].done = nullptr;
    }
    for (int i = 0; i < kRing; ++i) {
        if (hipEventCreateWithFlags(&c->ring[i].exp_ready, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&c->ring[i].done, hipEventDisableTiming) != hipSuccess) {
            destroy_events(c);
            delete c;
            return SALI_ERR_HIP;
        }
    }

    uint16_t lut[256 + 4096];
    fill_luts(lut, lut + 256);
    if (hipMemcpy(c->tables + c->tl.lut, lut, sizeof(lut), hipMemcpyHostToDevice) != hipSuccess ||
        sali_reset(c, nullptr) != SALI_OK || hipStreamSynchronize(nullptr) != hipSuccess) {
        sali_destroy(c);
        return SALI_ERR_HIP;
    }
    *out = c;
    return SALI_OK;
}

void sali_destroy(sali_ctx* ctx) {
    if (ctx == nullptr) return;
    destroy_events(ctx);
    delete ctx;
}

int sali_reset(sali_ctx* c, void* stream) {
    if (c == nullptr) return SALI_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int n = c->cfg.max_frames > kTokens ? c->cfg.max_frames : kTokens;
    LanePtrArray lanes;
    for (int l = 0; l < kLanes; ++l) lanes.lane[l] = c->lane_ptrs(l);
    // the adaptive thresholds start from the configured ones, on the 2^-16 lattice
    auto lattice = [](float x) { return (int)floorf(fminf(fmaxf(x, 0.0f), 1.0f) * 65536.0f); };
    hipLaunchKernelGGL(k_reset, dim3((n + 255) / 256), dim3(256), 0, s, c->cursors(), c->rows(), c->cfg.max_frames,
                       lanes, lattice(c->cfg.tau_high), lattice(c->cfg.tau_med), lattice(c->cfg.tau_low));
    SALI_TRY(hipGetLastError());
    c->n_analysed = 0;
    c->last_frame_id = -1;
    for (int l = 0; l < kLanes; ++l) c->lane_uses[l] = 0;
    for (int i = 0; i < kRing; ++i) c->ring[i].frame_id = -1;
    return SALI_OK;
}

int sali_set_gate_thresholds(sali_ctx* c, float tau_t, float theta_r) {
    if (c == nullptr) return SALI_ERR_NULL;
    if (!(tau_t >= 0.0f) || !(theta_r >= 0.0f)) return SALI_ERR_CONFIG;
    c->cfg.tau_t = tau_t;
    c->cfg.theta_r = theta_r;
    return SALI_OK;
}

int sali_set_tier_params(sali_ctx* c, int32_t tier_mode, float tau_high, float tau_med, float tau_low, int32_t k_fp16,
                         int32_t k_int8, int32_t k_int4) {
    if (c == nullptr) return SALI_ERR_NULL;
    sali_config trial = c->cfg;
    trial.tier_mode = tier_mode;
    trial.tau_high = tau_high;
    trial.tau_med = tau_med;
    trial.tau_low = tau_low;
    trial.k_fp16 = k_fp16;
    trial.k_int8 = k_int8;
    trial.k_int4 = k_int4;
    const int rc = check_config(&trial);
    if (rc != SALI_OK) return rc;
    c->cfg = trial;
    return SALI_OK;
}

int sali_flow_score(sali_ctx* c, const uint8_t* d_prev_rgb, const uint8_t* d_cur_rgb, float* d_flow_uv_or_null,
                    float* d_patch_motion576, sali_gate* d_gate_out, void* stream) {
    if (c == nullptr || d_prev_rgb == nullptr || d_cur_rgb == nullptr || d_patch_motion576 == nullptr ||
        d_gate_out == nullptr)
        return SALI_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    BatchPlan pa = {}, pb = {};
    pa.n = pb.n = 1;
    pa.slot[0] = kStepSlots;
    pa.prev_slot[0] = -1;
    pb.slot[0] = kStepSlots + 1;
    pb.prev_slot[0] = kStepSlots;
    int rc = enqueue_gray(c, &d_prev_rgb, pa, s);
    if (rc == SALI_OK) rc = enqueue_expansion(c, pa, s);
    if (rc == SALI_OK) rc = enqueue_gray(c, &d_cur_rgb, pb, s);
    if (rc == SALI_OK) rc = enqueue_expansion(c, pb, s);
    if (rc != SALI_OK) return rc;
    const float2* flow = nullptr;
    rc = enqueue_flow(c, pb, &flow, s);
    if (rc != SALI_OK) return rc;
    SALI_TRY(launch_patch_gate(flow, c->cfg.src_h, c->cfg.src_w, c->cfg.tau_t, c->cfg.theta_r, d_patch_motion576,
                               d_gate_out, &c->lane_ptrs(0).counters->patch_done, d_flow_uv_or_null, s));
    return SALI_OK;
}

int sali_saliency_pool(sali_ctx* c, const uint8_t* d_rgb, uint8_t* d_salmap_or_null, float* d_scores576,
                       void* stream) {
    if (c == nullptr || d_rgb == nullptr || d_scores576 == nullptr) return SALI_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    BatchPlan bp = {};
    bp.n = 1;
    bp.parity[0] = c->lane_uses[0]++ & 1u;
    int rc = enqueue_saliency(c, &d_rgb, bp, nullptr, s);
    if (rc == SALI_OK) rc = enqueue_pool(c, bp, d_scores576, d_salmap_or_null, nullptr, nullptr, s);
    return rc;
}

int sali_kv_compress(sali_ctx* c, const void* d_kv_fp16, const float* d_scores576, int32_t frame_id, void* stream) {
    if (c == nullptr || d_kv_fp16 == nullptr || d_scores576 == nullptr) return SALI_ERR_NULL;
    if (frame_id < 0 || frame_id >= c->cfg.max_frames) return SALI_ERR_SHAPE;
    if (!aligned16(d_kv_fp16)) return SALI_ERR_ALIGN;
    if (c->cfg.budget_tokens > 0 && frame_id <= c->last_frame_id) return SALI_ERR_STATE;
    if (frame_id > c->last_frame_id) c->last_frame_id = frame_id;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SALI_TRY(launch_tier(d_scores576, nullptr, tier_params(c->cfg), frame_id, c->rows(), c->tier(frame_id),
                         c->slot(frame_id), c->order(frame_id), c->cursors(), c->pools, c->cfg.budget_tokens,
                         c->cfg.tiles_per_frame > 1 ? c->cfg.tiles_per_frame : 1, s));
    return enqueue_pack(c, &d_kv_fp16, frame_id, 1, s);
}

int sali_kv_decompress_batch(sali_ctx* c, int32_t first_frame_id, int32_t n_frames, void* const* d_kv_fp16_out_frames,
                             uint8_t* d_valid_or_null, void* stream) {
    if (c == nullptr || d_kv_fp16_out_frames == nullptr) return SALI_ERR_NULL;
    if (n_frames < 1 || n_frames > kMaxBatch) return SALI_ERR_SHAPE;
    if (first_frame_id < 0 || (long long)first_frame_id + n_frames > c->cfg.max_frames) return SALI_ERR_SHAPE;
    KvBatch out = {};
    for (int i = 0; i < n_frames; ++i) {
        if (d_kv_fp16_out_frames[i] == nullptr) return SALI_ERR_NULL;
        if (!aligned16(d_kv_fp16_out_frames[i])) return SALI_ERR_ALIGN;
        out.kv[i] = d_kv_fp16_out_frames[i];
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t* ev = c->prof[SALI_PROF_UNPACK];
    if (ev[0] != nullptr) SALI_TRY(hipEventRecord(ev[0], s));
    SALI_TRY(launch_unpack(c->rows(), first_frame_id, c->tb<uint16_t>(c->tl.order), c->pools, out, n_frames,
                           d_valid_or_null, c->cursors(), c->n_planes, s));
    if (ev[1] != nullptr) SALI_TRY(hipEventRecord(ev[1], s));
    ev[0] = ev[1] = nullptr;
    return SALI_OK;
}

int sali_kv_decompress(sali_ctx* c, int32_t frame_id, void* d_kv_fp16_out, uint8_t* d_valid576_or_null,
                       void* stream) {
    if (c == nullptr || d_kv_fp16_out == nullptr) return SALI_ERR_NULL;
    return sali_kv_decompress_batch(c, frame_id, 1, &d_kv_fp16_out, d_valid576_or_null, stream);
}

int sali_attend_decode_gqa(sali_ctx* c, int32_t layer, const void* d_q_fp16, int32_t q_per_kv, int32_t frame_lo,
                           int32_t frame_hi, float softmax_scale, float* d_out, float* d_lse_or_null, void* stream) {
    if (c == nullptr || d_q_fp16 == nullptr || d_out == nullptr) return SALI_ERR_NULL;
    if (layer < 0 || layer >= c->cfg.n_layers) return SALI_ERR_SHAPE;
    if (q_per_kv != 1 && q_per_kv != 2 && q_per_kv != 4 && q_per_kv != 8 && !(q_per_kv > kAttnMaxQPerKv && q_per_kv <= 64))
        return SALI_ERR_SHAPE;
    if (frame_lo < 0 || frame_hi < frame_lo || frame_hi > c->cfg.max_frames) return SALI_ERR_SHAPE;
    if (!aligned16(d_q_fp16)) return SALI_ERR_ALIGN;
    if (!(softmax_scale == softmax_scale)) return SALI_ERR_CONFIG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t* ev = c->prof[SALI_PROF_ATTEND];
    const hipError_t e = launch_attend(c->rows(), c->pools, layer, c->cfg.n_heads, q_per_kv, d_q_fp16, frame_lo,
                                       frame_hi, softmax_scale, c->sc<float>(c->sl.attn_partial), d_out,
                                       d_lse_or_null, ev[0], ev[1], s);
    ev[0] = ev[1] = nullptr;
    return e == hipSuccess ? SALI_OK : SALI_ERR_HIP;
}

int sali_attend_decode(sali_ctx* c, int32_t layer, const void* d_q_fp16, int32_t frame_lo, int32_t frame_hi,
                       float softmax_scale, float* d_out, float* d_lse_or_null, void* stream) {
    return sali_attend_decode_gqa(c, layer, d_q_fp16, 1, frame_lo, frame_hi, softmax_scale, d_out, d_lse_or_null,
                                  stream);
}

int sali_attend_decode_static(sali_ctx* c, int32_t layer, const void* d_q_fp16, int32_t frame_lo, int32_t frame_hi,
                              float softmax_scale, float* d_out, float* d_lse_or_null, void* stream) {
    if (c == nullptr || d_q_fp16 == nullptr || d_out == nullptr) return SALI_ERR_NULL;
    if (c->cfg.n_heads > SALI_STATIC_ATTEND_MAX_HEADS) return SALI_ERR_SHAPE;      // the array holds no more
    if (layer < 0 || layer >= c->cfg.n_layers) return SALI_ERR_SHAPE;
    if (frame_lo < 0 || frame_hi < frame_lo || frame_hi > c->cfg.max_frames) return SALI_ERR_SHAPE;
    if (!aligned16(d_q_fp16)) return SALI_ERR_ALIGN;
    if (!(softmax_scale == softmax_scale)) return SALI_ERR_CONFIG;
    int dev = -1;
    SALI_TRY(hipGetDevice(&dev));
    if (dev != c->device || c->static_scratch == nullptr) return SALI_ERR_STATE;
    // every partial the merge kernel reads is written by the main kernel of the same call (one per
    // block, empty blocks included), so nothing of the previous call's contents has to be cleared
    const hipError_t e = launch_attend(c->rows(), c->pools, layer, c->cfg.n_heads, 1, d_q_fp16, frame_lo, frame_hi,
                                       softmax_scale, c->static_scratch, d_out, d_lse_or_null, nullptr, nullptr,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SALI_OK : SALI_ERR_HIP;
}

int sali_analyze_batch(sali_ctx* c, const uint8_t* const* d_rgb_frames, int32_t first_frame_id, int32_t n_frames,
                       void* stream) {
    if (c == nullptr || d_rgb_frames == nullptr) return SALI_ERR_NULL;
    if (n_frames < 1 || n_frames > kMaxBatch) return SALI_ERR_SHAPE;
    if (first_frame_id < 0 || (long long)first_frame_id + n_frames > c->cfg.max_frames) return SALI_ERR_SHAPE;
    for (int i = 0; i < n_frames; ++i)
        if (d_rgb_frames[i] == nullptr) return SALI_ERR_NULL;
    if (c->cfg.budget_tokens > 0 && first_frame_id <= c->last_frame_id) return SALI_ERR_STATE;
    // tiled frames come whole: entries t T .. t T + T - 1 in one call, and analysis number = entry number
    // modulo T, so that an entry's predecessor (the same tile of the frame before) is T analyses back
    const int tiles = c->cfg.tiles_per_frame > 1 ? c->cfg.tiles_per_frame : 1;
    if (first_frame_id % tiles != 0 || n_frames % tiles != 0) return SALI_ERR_SHAPE;
    if (first_frame_id + n_frames - 1 > c->last_frame_id) c->last_frame_id = first_frame_id + n_frames - 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned n0 = c->n_analysed;                  // analysis number of the batch's first frame
    const unsigned n_last = n0 + (unsigned)n_frames - 1u;
    BatchPlan bp = {};
    bp.n = n_frames;
    for (int i = 0; i < n_frames; ++i) {
        const unsigned n = n0 + (unsigned)i;
        bp.lane[i] = (int)(n % kLanes);
        bp.slot[i] = (int)(n % kStepSlots);
        bp.prev_slot[i] = n >= (unsigned)tiles ? (int)((n - (unsigned)tiles) % kStepSlots) : -1;
        bp.parity[i] = c->lane_uses[bp.lane[i]]++ & 1u;      // alternates per saliency pass in the lane
    }
    const AnalysisRecord* prev = n0 >= 1 ? &c->ring[c->ring[(n0 - 1) % kRing].batch_last] : nullptr;
    int rc;
    // A lane's scratch and expansion slot were last used by the analysis kLanes before (the slot
    // was read last by that one's successor's flow, which finished before it in tier order); tier
    // order also means the latest of them finishing implies that the others have.
    if (n_last >= (unsigned)kLanes) {
        const AnalysisRecord& old = c->ring[c->ring[(n_last - kLanes) % kRing].batch_last];
        rc = wait_unless_same(s, old.stream, old.done);
        if (rc != SALI_OK) return rc;
    }
    // the temporal filter first: gray, pyramid + expansion, flow, per-patch motion
    rc = enqueue_gray(c, d_rgb_frames, bp, s);
    if (rc == SALI_OK) rc = enqueue_expansion(c, bp, s);
    if (rc != SALI_OK) return rc;
    // the batch's events live in the ring entry of its last frame
    AnalysisRecord& rec = c->ring[n_last % kRing];
    SALI_TRY(hipEventRecord(rec.exp_ready, s));
    const float2* flow[kMaxBatch];
    if (prev != nullptr) {
        rc = wait_unless_same(s, prev->stream, prev->exp_ready);
        if (rc != SALI_OK) return rc;
    }
    rc = enqueue_flow(c, bp, flow, s);
    if (rc == SALI_OK) rc = enqueue_motion(c, bp, flow, s);
    // then the spatial filter, for the frames the reuse rule does not find redundant (Algorithm 1: a
    // redundant frame bypasses it): every kernel from here on evaluates the rule from the motions
    if (rc == SALI_OK) rc = enqueue_saliency(c, d_rgb_frames, bp, flow, s);
    if (rc != SALI_OK) return rc;
    if (prev != nullptr) {
        // tiers are handed out in frame order: the cursors must have seen the previous frame
        rc = wait_unless_same(s, prev->stream, prev->done);
        if (rc != SALI_OK) return rc;
    }
    // pooling, then gate and tiers
    const TierLaunch tl = tier_launch(c, first_frame_id);
    rc = enqueue_pool(c, bp, nullptr, nullptr, &tl, flow, s);
    if (rc != SALI_OK) return rc;
    SALI_TRY(hipEventRecord(rec.done, s));
    for (int i = 0; i < kRing; ++i)
        if (c->ring[i].frame_id >= first_frame_id && c->ring[i].frame_id < first_frame_id + n_frames)
            c->ring[i].frame_id = -1;      // an older analysis under the same id
    for (int i = 0; i < n_frames; ++i) {
        AnalysisRecord& r = c->ring[(n0 + (unsigned)i) % kRing];
        r.frame_id = first_frame_id + i;
        r.stream = s;
        r.batch_last = (int)(n_last % kRing);
    }
    c->n_analysed = n_last + 1u;
    return SALI_OK;
}

int sali_analyze(sali_ctx* c, const uint8_t* d_rgb, int32_t frame_id, void* stream) {
    if (c == nullptr || d_rgb == nullptr) return SALI_ERR_NULL;
    return sali_analyze_batch(c, &d_rgb, frame_id, 1, stream);
}

int sali_store_batch(sali_ctx* c, const void* const* d_kv_frames, int32_t first_frame_id, int32_t n_frames,
                     void* stream) {
    if (c == nullptr || d_kv_frames == nullptr) return SALI_ERR_NULL;
    if (n_frames < 1 || n_frames > kMaxBatch) return SALI_ERR_SHAPE;
    if (first_frame_id < 0 || (long long)first_frame_id + n_frames > c->cfg.max_frames) return SALI_ERR_SHAPE;
    for (int i = 0; i < n_frames; ++i) {
        if (d_kv_frames[i] == nullptr) return SALI_ERR_NULL;
        if (!aligned16(d_kv_frames[i])) return SALI_ERR_ALIGN;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // every frame must have been analysed recently; wait once per batch of analyses
    const AnalysisRecord* waits[kMaxBatch];
    int n_waits = 0;
    for (int f = 0; f < n_frames; ++f) {
        const AnalysisRecord* rec = nullptr;
        for (int i = 0; i < kRing; ++i)
            if (c->ring[i].frame_id == first_frame_id + f) rec = &c->ring[i];
        if (rec == nullptr) return SALI_ERR_STATE;      // not analysed (or too long ago)
        const AnalysisRecord* ev = &c->ring[rec->batch_last];
        if (n_waits == 0 || waits[n_waits - 1] != ev) waits[n_waits++] = ev;
    }
    for (int i = 0; i < n_waits; ++i) {
        const int rc = wait_unless_same(s, waits[i]->stream, waits[i]->done);
        if (rc != SALI_OK) return rc;
    }
    return enqueue_pack(c, d_kv_frames, first_frame_id, n_frames, s);
}

int sali_store(sali_ctx* c, const void* d_kv, int32_t frame_id, void* stream) {
    if (c == nullptr || d_kv == nullptr) return SALI_ERR_NULL;
    return sali_store_batch(c, &d_kv, frame_id, 1, stream);
}

int sali_step(sali_ctx* c, const uint8_t* d_rgb_t, const void* d_kv_t, int32_t frame_id, void* stream) {
    if (c == nullptr || d_rgb_t == nullptr || d_kv_t == nullptr) return SALI_ERR_NULL;
    if (!aligned16(d_kv_t)) return SALI_ERR_ALIGN;
    const int rc = sali_analyze(c, d_rgb_t, frame_id, stream);
    if (rc != SALI_OK) return rc;
    return sali_store(c, d_kv_t, frame_id, stream);
}

int sali_step_batch(sali_ctx* c, const uint8_t* const* d_rgb_frames, const void* const* d_kv_frames,
                    int32_t first_frame_id, int32_t n_frames, void* stream) {
    if (c == nullptr || d_rgb_frames == nullptr || d_kv_frames == nullptr) return SALI_ERR_NULL;
    if (n_frames < 1 || n_frames > kMaxBatch) return SALI_ERR_SHAPE;
    for (int i = 0; i < n_frames; ++i) {
        if (d_kv_frames[i] == nullptr) return SALI_ERR_NULL;
        if (!aligned16(d_kv_frames[i])) return SALI_ERR_ALIGN;
    }
    const int rc = sali_analyze_batch(c, d_rgb_frames, first_frame_id, n_frames, stream);
    if (rc != SALI_OK) return rc;
    return sali_store_batch(c, d_kv_frames, first_frame_id, n_frames, stream);
}

int sali_step_pipelined(sali_ctx* c, const uint8_t* d_rgb_next_or_null, int32_t next_frame_id,
                        const void* d_kv_or_null, int32_t frame_id, void* image_stream, void* kv_stream) {
    if (c == nullptr) return SALI_ERR_NULL;
    if (d_kv_or_null != nullptr && !aligned16(d_kv_or_null)) return SALI_ERR_ALIGN;
    if (d_rgb_next_or_null != nullptr) {
        const int rc = sali_analyze(c, d_rgb_next_or_null, next_frame_id, image_stream);
        if (rc != SALI_OK) return rc;
    }
    if (d_kv_or_null != nullptr) return sali_store(c, d_kv_or_null, frame_id, kv_stream);
    return SALI_OK;
}

int sali_read_frame_table(sali_ctx* c, sali_frame_row* h_rows, int32_t first, int32_t count, void* stream) {
    if (c == nullptr || h_rows == nullptr) return SALI_ERR_NULL;
    if (first < 0 || count < 0 || (long long)first + count > c->cfg.max_frames) return SALI_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (count > 0)
        SALI_TRY(hipMemcpyAsync(h_rows, c->rows() + first, (size_t)count * sizeof(sali_frame_row),
                                hipMemcpyDeviceToHost, s));
    SALI_TRY(hipStreamSynchronize(s));
    return SALI_OK;
}

int sali_read_frame_tiers(sali_ctx* c, int32_t frame_id, uint8_t* h_tier576, uint16_t* h_slot576, void* stream) {
    if (c == nullptr || h_tier576 == nullptr || h_slot576 == nullptr) return SALI_ERR_NULL;
    if (frame_id < 0 || frame_id >= c->cfg.max_frames) return SALI_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SALI_TRY(hipMemcpyAsync(h_tier576, c->tier(frame_id), kTokens, hipMemcpyDeviceToHost, s));
    SALI_TRY(hipMemcpyAsync(h_slot576, c->slot(frame_id), kTokens * sizeof(uint16_t), hipMemcpyDeviceToHost, s));
    SALI_TRY(hipStreamSynchronize(s));
    return SALI_OK;
}

int sali_read_last_step(sali_ctx* c, float* h_patch_motion576, sali_gate* h_gate, float* h_scores576, void* stream) {
    if (c == nullptr) return SALI_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const LanePtrs lp = c->lane_ptrs(c->n_analysed == 0 ? 0 : (int)((c->n_analysed - 1) % kLanes));
    if (h_patch_motion576 != nullptr)
        SALI_TRY(hipMemcpyAsync(h_patch_motion576, lp.dp, kTokens * sizeof(float), hipMemcpyDeviceToHost, s));
    if (h_gate != nullptr) SALI_TRY(hipMemcpyAsync(h_gate, lp.gate, sizeof(sali_gate), hipMemcpyDeviceToHost, s));
    if (h_scores576 != nullptr)
        SALI_TRY(hipMemcpyAsync(h_scores576, lp.scores, kTokens * sizeof(float), hipMemcpyDeviceToHost, s));
    SALI_TRY(hipStreamSynchronize(s));
    return SALI_OK;
}

int sali_read_analysis(sali_ctx* c, int32_t frame_id, float* h_patch_motion576, sali_gate* h_gate, float* h_scores576,
                       void* stream) {
    if (c == nullptr) return SALI_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int slot = -1;
    for (int i = 0; i < kRing; ++i)
        if (c->ring[i].frame_id == frame_id) slot = i;
    if (slot < 0 || c->n_analysed == 0) return SALI_ERR_STATE;
    // analysis number of that ring entry: the latest n < n_analysed with n % kRing == slot; its
    // scratch copy has been handed to analysis n + kLanes if that one was issued already
    const unsigned last = c->n_analysed - 1u;
    const unsigned n = last - ((last + (unsigned)kRing - (unsigned)slot) % (unsigned)kRing);
    if (c->n_analysed - n > (unsigned)kLanes) return SALI_ERR_STATE;
    const AnalysisRecord& ev = c->ring[c->ring[slot].batch_last];
    const int rc = wait_unless_same(s, ev.stream, ev.done);
    if (rc != SALI_OK) return rc;
    const LanePtrs lp = c->lane_ptrs((int)(n % kLanes));
    if (h_patch_motion576 != nullptr)
        SALI_TRY(hipMemcpyAsync(h_patch_motion576, lp.dp, kTokens * sizeof(float), hipMemcpyDeviceToHost, s));
    if (h_gate != nullptr) SALI_TRY(hipMemcpyAsync(h_gate, lp.gate, sizeof(sali_gate), hipMemcpyDeviceToHost, s));
    if (h_scores576 != nullptr)
        SALI_TRY(hipMemcpyAsync(h_scores576, lp.scores, kTokens * sizeof(float), hipMemcpyDeviceToHost, s));
    SALI_TRY(hipStreamSynchronize(s));
    return SALI_OK;
}

int sali_set_profile_events(sali_ctx* c, int which, void* start_event, void* stop_event) {
    if (c == nullptr) return SALI_ERR_NULL;
    if (which != SALI_PROF_PACK && which != SALI_PROF_UNPACK && which != SALI_PROF_ATTEND) return SALI_ERR_SHAPE;
    c->prof[which][0] = static_cast<hipEvent_t>(start_event);
    c->prof[which][1] = static_cast<hipEvent_t>(stop_event);
    return SALI_OK;
}

int sali_get_status(sali_ctx* c, uint32_t* h_flags, void* stream) {
    if (c == nullptr || h_flags == nullptr) return SALI_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SALI_TRY(hipMemcpyAsync(h_flags, &c->cursors()->status, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    SALI_TRY(hipStreamSynchronize(s));
    return SALI_OK;
}

const char* sali_error_string(int code) {
    switch (code) {
        case SALI_OK: return "ok";
        case SALI_ERR_NULL: return "null pointer";
        case SALI_ERR_SHAPE: return "index or size out of range";
        case SALI_ERR_ALIGN: return "misaligned pointer";
        case SALI_ERR_CONFIG: return "invalid configuration";
        case SALI_ERR_STATE: return "invalid state";
        case SALI_ERR_HIP: return "HIP runtime error";
        default: return "unknown";
    }
}

}  // extern "C"
