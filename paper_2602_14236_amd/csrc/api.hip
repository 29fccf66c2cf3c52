// C ABI of libsali: context management, argument checks and the per-call kernel chains.
// Every step of the method runs in the kernels of kv_kernels.hip, saliency_kernels.hip and
// flow_kernels.hip; this file only validates, lays out the caller's buffers and enqueues.

#include <math.h>
#include <new>
#include <string.h>

#include "sali_internal.h"

namespace sali {

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Image-side scratch exists in kLanes copies so that the analyses of consecutive frames can be in
// flight at once on different streams; polynomial expansions live in a ring one longer than that
// (a frame's flow reads its predecessor's expansion), plus two slots for the stand-alone flow call.
constexpr int kLanes = SALI_ANALYSIS_LANES;
constexpr int kStepSlots = kLanes + 1;
constexpr int kExpSlots = kStepSlots + 2;
constexpr int kRing = 8;              // bookkeeping of the most recent analyses

struct LaneLayout {
    size_t y8, pyr, flow[2], cls, var, parent, msum, dp, scores, gate, counters;
};

struct ScratchLayout {
    LaneLayout lane[kLanes];
    size_t expA[kExpSlots], expB[kExpSlots];
    size_t total;
};

struct TableLayout {
    size_t lut, cursors, rows, tier, slot, order, total;      // lut = lin[256] followed by fl[4096]
};

struct LaneCounters {
    uint32_t patch_done;      // arrival counter of the patch-motion kernel (self-resetting)
    uint32_t pool_done;       // arrival counter of the pooling kernel (self-resetting)
};

int check_config(const sali_config* c) {
    if (c == nullptr) return SALI_ERR_NULL;
    if (c->grid != kGrid || c->head_dim != kHeadDim || c->group != kGroup) return SALI_ERR_CONFIG;
    if (c->src_h < kGrid || c->src_w < kGrid || c->src_h > 16384 || c->src_w > 16384) return SALI_ERR_CONFIG;
    if (c->flow_levels < 1 || c->flow_levels > kMaxLevels || c->flow_iters < 1 || c->flow_iters > kMaxIters)
        return SALI_ERR_CONFIG;
    if (!(c->tau_t >= 0.0f) || !(c->theta_r >= 0.0f)) return SALI_ERR_CONFIG;
    if (c->canny_lo < 1 || c->canny_hi < c->canny_lo || c->canny_hi > 1442) return SALI_ERR_CONFIG;
    if (c->tier_mode != 0 && c->tier_mode != 1) return SALI_ERR_CONFIG;
    if (c->tier_mode == 0) {
        if (!(c->tau_low <= c->tau_med) || !(c->tau_med <= c->tau_high)) return SALI_ERR_CONFIG;
    } else {
        if (c->k_fp16 < 0 || c->k_int8 < 0 || c->k_int4 < 0 ||
            (long long)c->k_fp16 + c->k_int8 + c->k_int4 > kTokens)
            return SALI_ERR_CONFIG;
    }
    if (c->n_layers < 1 || c->n_heads < 1 || (long long)c->n_layers * 2 * c->n_heads > 65535) return SALI_ERR_CONFIG;
    if (c->cap_fp16 < 0 || c->cap_int8 < 0 || c->cap_int4 < 0) return SALI_ERR_CONFIG;
    if (c->cap_fp16 > 0x7FFFFFFFll || c->cap_int8 > 0x7FFFFFFFll || c->cap_int4 > 0x7FFFFFFFll) return SALI_ERR_CONFIG;
    if (c->max_frames < 1 || c->max_frames > (1 << 24)) return SALI_ERR_CONFIG;
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
    }
    for (int i = 0; i < kExpSlots; ++i) {
        s.expA[i] = take(px * sizeof(float4));
        s.expB[i] = take(px * sizeof(float2));
    }
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

__global__ void k_reset(Cursors* cur, sali_frame_row* rows, int max_frames, LanePtrArray lanes) {
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
            LaneCounters z = {0u, 0u};
            *lanes.lane[l].counters = z;
        }
    }
    if (i == 0) {
        Cursors c = {};
        c.last_src = -1;
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
    unsigned n_analysed;      // analyses since create / reset; analysis n uses lane n % kLanes
    unsigned lane_uses[kLanes];   // saliency passes run in each lane; the parity selects the frame-sum accumulator
    AnalysisRecord ring[kRing];
    hipEvent_t prof[2][2];    // [SALI_PROF_*][start, stop], armed for one launch

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

// gray (+ saliency pre-pass) of one frame in lane `lane`; msum_parity selects the accumulator of
// the colour-variance frame sum (the other one is cleared for the lane's next use)
int enqueue_prep(sali_ctx* c, const uint8_t* d_rgb, int lane, bool with_saliency, unsigned msum_parity,
                 hipStream_t s) {
    const sali_config& cfg = c->cfg;
    const LaneLayout& L = c->sl.lane[lane];
    unsigned long long* msum = c->sc<unsigned long long>(L.msum);
    unsigned long long* acc = with_saliency ? msum + (msum_parity & 1u) : nullptr;
    unsigned long long* clr = with_saliency ? msum + ((msum_parity + 1u) & 1u) : nullptr;
    SALI_TRY(launch_prep(d_rgb, cfg.src_h, cfg.src_w, with_saliency, c->sc<uint8_t>(L.y8), c->sc<uint8_t>(L.cls),
                         c->sc<uint32_t>(L.var), c->sc<uint32_t>(L.parent), acc, clr, c->tb<uint16_t>(c->tl.lut),
                         cfg.canny_lo * cfg.canny_lo, cfg.canny_hi * cfg.canny_hi, s));
    // cross-tile hysteresis (a kernel boundary is the cheapest device-wide ordering there is)
    if (with_saliency)
        SALI_TRY(launch_union(c->sc<uint8_t>(L.cls), c->sc<uint32_t>(L.parent), cfg.src_h, cfg.src_w, s));
    return SALI_OK;
}

// pyramid and polynomial expansion of the lane's gray image into expansion slot `slot`
int enqueue_expansion(sali_ctx* c, int lane, int slot, hipStream_t s) {
    const LaneLayout& L = c->sl.lane[lane];
    float* pyr = c->sc<float>(L.pyr);
    const LevelGeom& g = c->geom;
    if (g.levels <= 3) {
        SALI_TRY(launch_expand(c->sc<uint8_t>(L.y8), g, c->fw, c->sc<float4>(c->sl.expA[slot]),
                               c->sc<float2>(c->sl.expB[slot]), s));
        return SALI_OK;
    }
    for (int l = 1; l < g.levels; ++l) {
        SALI_TRY(launch_pyr_down(l == 1 ? c->sc<uint8_t>(L.y8) : nullptr, l == 1 ? nullptr : pyr + g.off[l - 1],
                                 g.h[l - 1], g.w[l - 1], pyr + g.off[l], g.h[l], g.w[l], s));
    }
    SALI_TRY(launch_polyexp(c->sc<uint8_t>(L.y8), pyr, g, c->fw, c->sc<float4>(c->sl.expA[slot]),
                            c->sc<float2>(c->sl.expB[slot]), s));
    return SALI_OK;
}

// coarse-to-fine displacement estimation between expansion slots; result in *result_buf
int enqueue_flow(sali_ctx* c, int lane, int slot_prev, int slot_cur, const float2** result_buf, hipStream_t s) {
    const LevelGeom& g = c->geom;
    const LaneLayout& L = c->sl.lane[lane];
    float2* buf[2] = {c->sc<float2>(L.flow[0]), c->sc<float2>(L.flow[1])};
    const float4* A1 = c->sc<float4>(c->sl.expA[slot_prev]);
    const float2* b1 = c->sc<float2>(c->sl.expB[slot_prev]);
    const float4* A2 = c->sc<float4>(c->sl.expA[slot_cur]);
    const float2* b2 = c->sc<float2>(c->sl.expB[slot_cur]);
    int cur = 0;            // buffer holding the latest estimate
    bool have = false;
    for (int l = g.levels - 1; l >= 0; --l) {
        for (int it = 0; it < c->cfg.flow_iters; ++it) {
            int mode;
            int ch = 0, cw = 0;
            if (it > 0) mode = 2;
            else if (!have) mode = 0;
            else { mode = 1; ch = g.h[l + 1]; cw = g.w[l + 1]; }
            SALI_TRY(launch_flow_iter(A1 + g.off[l], b1 + g.off[l], A2 + g.off[l], b2 + g.off[l], buf[cur],
                                      buf[cur ^ 1], g.h[l], g.w[l], ch, cw, mode, c->fw, s));
            cur ^= 1;
            have = true;
        }
    }
    *result_buf = buf[cur];
    return SALI_OK;
}

// pooling of the lane's saliency pre-pass.  With `tier` (the chained step) the kernel also reduces
// `flow` (NULL for the first frame of a sequence) to per-patch motion, evaluates the gate and writes
// the frame-table row with tiers and compaction indices.
int enqueue_pool(sali_ctx* c, int lane, unsigned msum_parity, float* d_scores, uint8_t* d_salmap,
                 const TierLaunch* tier, const float2* flow, hipStream_t s) {
    const LaneLayout& L = c->sl.lane[lane];
    const LanePtrs lp = c->lane_ptrs(lane);
    SALI_TRY(launch_pool(c->sc<uint8_t>(L.cls), c->sc<uint32_t>(L.parent), c->sc<uint32_t>(L.var),
                         c->sc<unsigned long long>(L.msum) + (msum_parity & 1u), c->cfg.src_h, c->cfg.src_w, d_scores,
                         d_salmap, tier, flow, c->cfg.tau_t, c->cfg.theta_r, lp.dp, lp.gate, &lp.counters->pool_done,
                         s));
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
    return t;
}

// the storage kernel of frame `frame_id`; its frame-table row and order list must be in place
int enqueue_pack(sali_ctx* c, const void* d_kv, int frame_id, hipStream_t s) {
    hipEvent_t* ev = c->prof[SALI_PROF_PACK];
    if (ev[0] != nullptr) SALI_TRY(hipEventRecord(ev[0], s));
    SALI_TRY(launch_pack(d_kv, c->rows() + frame_id, c->order(frame_id), c->pools, c->cursors(), c->n_planes, s));
    if (ev[1] != nullptr) SALI_TRY(hipEventRecord(ev[1], s));
    ev[0] = ev[1] = nullptr;
    return SALI_OK;
}

// make stream `s` wait for `ev` unless the event was recorded on `s` itself
int wait_unless_same(hipStream_t s, hipStream_t recorded_on, hipEvent_t ev) {
    if (recorded_on != s) SALI_TRY(hipStreamWaitEvent(s, ev, 0));
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
    c->n_analysed = 0;
    for (int l = 0; l < kLanes; ++l) c->lane_uses[l] = 0;
    c->prof[0][0] = c->prof[0][1] = c->prof[1][0] = c->prof[1][1] = nullptr;
    for (int i = 0; i < kRing; ++i) {
        c->ring[i].frame_id = -1;
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
    hipLaunchKernelGGL(k_reset, dim3((n + 255) / 256), dim3(256), 0, s, c->cursors(), c->rows(), c->cfg.max_frames,
                       lanes);
    SALI_TRY(hipGetLastError());
    c->n_analysed = 0;
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

int sali_flow_score(sali_ctx* c, const uint8_t* d_prev_rgb, const uint8_t* d_cur_rgb, float* d_flow_uv_or_null,
                    float* d_patch_motion576, sali_gate* d_gate_out, void* stream) {
    if (c == nullptr || d_prev_rgb == nullptr || d_cur_rgb == nullptr || d_patch_motion576 == nullptr ||
        d_gate_out == nullptr)
        return SALI_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int lane = 0, slot_a = kStepSlots, slot_b = kStepSlots + 1;
    int rc = enqueue_prep(c, d_prev_rgb, lane, false, 0, s);
    if (rc == SALI_OK) rc = enqueue_expansion(c, lane, slot_a, s);
    if (rc == SALI_OK) rc = enqueue_prep(c, d_cur_rgb, lane, false, 0, s);
    if (rc == SALI_OK) rc = enqueue_expansion(c, lane, slot_b, s);
    if (rc != SALI_OK) return rc;
    const float2* flow = nullptr;
    rc = enqueue_flow(c, lane, slot_a, slot_b, &flow, s);
    if (rc != SALI_OK) return rc;
    SALI_TRY(launch_patch_gate(flow, c->cfg.src_h, c->cfg.src_w, c->cfg.tau_t, c->cfg.theta_r, d_patch_motion576,
                               d_gate_out, &c->lane_ptrs(lane).counters->patch_done, d_flow_uv_or_null, s));
    return SALI_OK;
}

int sali_saliency_pool(sali_ctx* c, const uint8_t* d_rgb, uint8_t* d_salmap_or_null, float* d_scores576,
                       void* stream) {
    if (c == nullptr || d_rgb == nullptr || d_scores576 == nullptr) return SALI_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int lane = 0;
    const unsigned parity = c->lane_uses[lane]++ & 1u;
    int rc = enqueue_prep(c, d_rgb, lane, true, parity, s);
    if (rc == SALI_OK) rc = enqueue_pool(c, lane, parity, d_scores576, d_salmap_or_null, nullptr, nullptr, s);
    return rc;
}

int sali_kv_compress(sali_ctx* c, const void* d_kv_fp16, const float* d_scores576, int32_t frame_id, void* stream) {
    if (c == nullptr || d_kv_fp16 == nullptr || d_scores576 == nullptr) return SALI_ERR_NULL;
    if (frame_id < 0 || frame_id >= c->cfg.max_frames) return SALI_ERR_SHAPE;
    if (!aligned16(d_kv_fp16)) return SALI_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SALI_TRY(launch_tier(d_scores576, nullptr, tier_params(c->cfg), frame_id, c->rows(), c->tier(frame_id),
                         c->slot(frame_id), c->order(frame_id), c->cursors(), c->pools, s));
    return enqueue_pack(c, d_kv_fp16, frame_id, s);
}

int sali_kv_decompress(sali_ctx* c, int32_t frame_id, void* d_kv_fp16_out, uint8_t* d_valid576_or_null,
                       void* stream) {
    if (c == nullptr || d_kv_fp16_out == nullptr) return SALI_ERR_NULL;
    if (frame_id < 0 || frame_id >= c->cfg.max_frames) return SALI_ERR_SHAPE;
    if (!aligned16(d_kv_fp16_out)) return SALI_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t* ev = c->prof[SALI_PROF_UNPACK];
    if (ev[0] != nullptr) SALI_TRY(hipEventRecord(ev[0], s));
    SALI_TRY(launch_unpack(c->rows(), frame_id, c->tb<uint16_t>(c->tl.order), c->pools, d_kv_fp16_out,
                           d_valid576_or_null, c->cursors(), c->n_planes, s));
    if (ev[1] != nullptr) SALI_TRY(hipEventRecord(ev[1], s));
    ev[0] = ev[1] = nullptr;
    return SALI_OK;
}

int sali_analyze(sali_ctx* c, const uint8_t* d_rgb, int32_t frame_id, void* stream) {
    if (c == nullptr || d_rgb == nullptr) return SALI_ERR_NULL;
    if (frame_id < 0 || frame_id >= c->cfg.max_frames) return SALI_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned n = c->n_analysed;
    const int lane = (int)(n % kLanes);
    const int slot = (int)(n % kStepSlots);
    const unsigned parity = c->lane_uses[lane]++ & 1u;      // alternates per saliency pass in the lane
    AnalysisRecord& rec = c->ring[n % kRing];
    const AnalysisRecord* prev = n >= 1 ? &c->ring[(n - 1) % kRing] : nullptr;
    int rc;
    // the lane's scratch and the expansion slot were last used by analysis n - kLanes (and read by
    // the flow of its successor, which finished before it in tier order)
    if (n >= (unsigned)kLanes) {
        const AnalysisRecord& old = c->ring[(n - kLanes) % kRing];
        rc = wait_unless_same(s, old.stream, old.done);
        if (rc != SALI_OK) return rc;
    }
    rc = enqueue_prep(c, d_rgb, lane, true, parity, s);
    if (rc == SALI_OK) rc = enqueue_expansion(c, lane, slot, s);
    if (rc != SALI_OK) return rc;
    SALI_TRY(hipEventRecord(rec.exp_ready, s));
    const LanePtrs lp = c->lane_ptrs(lane);
    const float2* flow = nullptr;
    if (prev != nullptr) {
        rc = wait_unless_same(s, prev->stream, prev->exp_ready);
        if (rc != SALI_OK) return rc;
        rc = enqueue_flow(c, lane, (int)((n - 1) % kStepSlots), slot, &flow, s);
        if (rc != SALI_OK) return rc;
        // tiers are handed out in frame order: the cursors must have seen the previous frame
        rc = wait_unless_same(s, prev->stream, prev->done);
        if (rc != SALI_OK) return rc;
    }
    // per-patch motion, gate, pooling, tiers: one launch (first frame: no flow, never redundant)
    const TierLaunch tl = tier_launch(c, frame_id);
    rc = enqueue_pool(c, lane, parity, lp.scores, nullptr, &tl, flow, s);
    if (rc != SALI_OK) return rc;
    SALI_TRY(hipEventRecord(rec.done, s));
    for (int i = 0; i < kRing; ++i)
        if (c->ring[i].frame_id == frame_id) c->ring[i].frame_id = -1;      // an older analysis under the same id
    rec.frame_id = frame_id;
    rec.stream = s;
    c->n_analysed = n + 1;
    return SALI_OK;
}

int sali_store(sali_ctx* c, const void* d_kv, int32_t frame_id, void* stream) {
    if (c == nullptr || d_kv == nullptr) return SALI_ERR_NULL;
    if (frame_id < 0 || frame_id >= c->cfg.max_frames) return SALI_ERR_SHAPE;
    if (!aligned16(d_kv)) return SALI_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const AnalysisRecord* rec = nullptr;
    for (int i = 0; i < kRing; ++i)
        if (c->ring[i].frame_id == frame_id) rec = &c->ring[i];
    if (rec == nullptr) return SALI_ERR_STATE;      // not analysed (or too long ago)
    const int rc = wait_unless_same(s, rec->stream, rec->done);
    if (rc != SALI_OK) return rc;
    return enqueue_pack(c, d_kv, frame_id, s);
}

int sali_step(sali_ctx* c, const uint8_t* d_rgb_t, const void* d_kv_t, int32_t frame_id, void* stream) {
    if (c == nullptr || d_rgb_t == nullptr || d_kv_t == nullptr) return SALI_ERR_NULL;
    if (!aligned16(d_kv_t)) return SALI_ERR_ALIGN;
    const int rc = sali_analyze(c, d_rgb_t, frame_id, stream);
    if (rc != SALI_OK) return rc;
    return sali_store(c, d_kv_t, frame_id, stream);
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

int sali_set_profile_events(sali_ctx* c, int which, void* start_event, void* stop_event) {
    if (c == nullptr) return SALI_ERR_NULL;
    if (which != SALI_PROF_PACK && which != SALI_PROF_UNPACK) return SALI_ERR_SHAPE;
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
