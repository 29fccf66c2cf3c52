// Tier assignment (Eq. 8 or top-k counts), compaction indices and frame-table row for one frame.
// Shared by the stand-alone tier kernel and by the pooling kernel.  Two parts: tier_rank (a whole
// block of exactly kTierThreads threads; everything that depends on the frame's scores only) and
// tier_commit (one thread; the part that depends on the pool cursors, so it runs in frame order).
// In tier_rank thread t owns tokens t, t + 256 and (for t < 64) t + 512, so the 64 tokens of
// "group" g = token / 64 sit in one wave.  Only comparisons and integer arithmetic: the result does
// not depend on floating-point contraction.
//
// Workgroups are kept at 256 threads on purpose: larger ones wait for many free wave slots on
// one compute unit and starve next to a bandwidth kernel that keeps every unit busy.
#pragma once

#include "sali_internal.h"

namespace sali {

constexpr int kTierThreads = 256;
constexpr int kTierSlots = (kTokens + kTierThreads - 1) / kTierThreads;      // tokens per thread (3)
constexpr int kTierGroups = kTokens / 64;                                    // 9

// what tier_rank hands to tier_commit
struct TierCounts {
    int32_t state;          // 0 = tiers assigned, 1 = redundant frame, 2 = a score was NaN,
                            // 3 = ranked only (adaptive thresholds: tiers are assigned in frame order)
    int32_t cnt[4];         // tokens per tier
    int32_t q[3];           // state 3: the frame's score quantiles at the target ranks, units of 2^-16
};

struct TierShared {
    uint4 key4[kTokens / 4];        // order-preserving integer image of the scores
    int group_cnt[kTierGroups][4];
    int part_rank[4][64];           // partial ranks of tokens 512..575, one row per wave
    int nan_flag;
    int q[3];                       // adaptive thresholds: quantiles found by the ranking
    int tau[3];                     // adaptive thresholds in force, units of 2^-16
};

// floor(clamp(x, 0, 1) * 2^16): scores and thresholds of the adaptive mode live on this lattice, so
// that the update rule is integer arithmetic
__device__ __forceinline__ int to_lattice(float x) {
    return (int)floorf(fminf(fmaxf(x, 0.0f), 1.0f) * 65536.0f);
}

// Number of tokens j in key blocks [j4_lo, j4_hi) (four keys per block) that precede token i in
// (key descending, index ascending) order; `me` = key of token i.  Blocks before the token's own
// 64-token group count with >=, blocks after it with >, and only the 16 blocks of the own group
// need the index test.  128-bit broadcast LDS reads, eight in flight.
__device__ __forceinline__ int tier_count_above(const TierShared& sh, uint32_t me, int i, int j4_lo, int j4_hi) {
    const int own0 = (i >> 6) * 16, own1 = own0 + 16;
    int rank = 0;
    const int a1 = own0 < j4_hi ? own0 : j4_hi;          // [j4_lo, a1): earlier groups
    const int b0 = own0 > j4_lo ? own0 : j4_lo;          // [b0, b1): own group
    const int b1 = own1 < j4_hi ? own1 : j4_hi;
    const int c0 = own1 > j4_lo ? own1 : j4_lo;          // [c0, j4_hi): later groups
#pragma unroll 8
    for (int j4 = j4_lo; j4 < a1; ++j4) {
        const uint4 v = sh.key4[j4];
        rank += (v.x >= me ? 1 : 0) + (v.y >= me ? 1 : 0) + (v.z >= me ? 1 : 0) + (v.w >= me ? 1 : 0);
    }
#pragma unroll 8
    for (int j4 = b0; j4 < b1; ++j4) {
        const uint4 v = sh.key4[j4];
        const int j = 4 * j4;
        rank += (v.x > me || (v.x == me && j < i)) ? 1 : 0;
        rank += (v.y > me || (v.y == me && j + 1 < i)) ? 1 : 0;
        rank += (v.z > me || (v.z == me && j + 2 < i)) ? 1 : 0;
        rank += (v.w > me || (v.w == me && j + 3 < i)) ? 1 : 0;
    }
#pragma unroll 8
    for (int j4 = c0; j4 < j4_hi; ++j4) {
        const uint4 v = sh.key4[j4];
        rank += (v.x > me ? 1 : 0) + (v.y > me ? 1 : 0) + (v.z > me ? 1 : 0) + (v.w > me ? 1 : 0);
    }
    return rank;
}

// Assigns tier, slot (rank inside the tier in token order) and the pool-order token list of one
// non-redundant frame.  Returns the per-tier counts (every thread gets the same value).
// The scores of the thread's tokens (0 past the end).  A step of its own so that a caller can ask for
// them early, together with other loads it has to wait for anyway.
struct TierScores {
    float s[kTierSlots];
};
__device__ __forceinline__ TierScores tier_load_scores(const float* scores) {
    TierScores v;
#pragma unroll
    for (int k = 0; k < kTierSlots; ++k) {
        const int i = (int)threadIdx.x + k * kTierThreads;
        v.s[k] = i < kTokens ? __hip_atomic_load(scores + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0f;
    }
    return v;
}

// Eq. 8 for the thread's tokens, inequalities as printed
__device__ __forceinline__ void tier_by_thresholds(const float* s, float tau_high, float tau_med, float tau_low, int* tier) {
#pragma unroll
    for (int k = 0; k < kTierSlots; ++k) {
        const int i = (int)threadIdx.x + k * kTierThreads;
        tier[k] = SALI_TIER_PRUNE;
        if (i >= kTokens) continue;
        if (s[k] > tau_low) tier[k] = SALI_TIER_INT4;
        if (s[k] > tau_med) tier[k] = SALI_TIER_INT8;
        if (s[k] > tau_high) tier[k] = SALI_TIER_FP16;
    }
}

// Compaction indices from the tiers of the thread's tokens; writes tier, slot and the pool-order token
// list and returns the per-tier counts (every thread gets the same value).  Whole block.
__device__ __forceinline__ TierCounts tier_finish(TierShared& sh, const int* tier, uint8_t* __restrict__ tier_out,
                                                  uint16_t* __restrict__ slot_out, uint16_t* __restrict__ order_out) {
    // slot = number of earlier tokens in the same tier: ballot inside the group + prefix over groups
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    TierCounts res = {};
    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int in_group[kTierSlots];
#pragma unroll
    for (int k = 0; k < kTierSlots; ++k) {
        const int i = tid + k * kTierThreads;
        const bool valid = i < kTokens;
        in_group[k] = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const unsigned long long m = __ballot(valid && tier[k] == t);
            if (valid && tier[k] == t) in_group[k] = __popcll(m & lt_mask);
            if (valid && lane == 0) sh.group_cnt[i >> 6][t] = __popcll(m);
        }
    }
    __syncthreads();
    int cnt[4] = {0, 0, 0, 0};
    int before[kTierSlots];
#pragma unroll
    for (int k = 0; k < kTierSlots; ++k) before[k] = 0;
    for (int g = 0; g < kTierGroups; ++g) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int c = sh.group_cnt[g][t];
            cnt[t] += c;
#pragma unroll
            for (int k = 0; k < kTierSlots; ++k) {
                const int i = tid + k * kTierThreads;
                if (g < (i >> 6) && t == tier[k]) before[k] += c;
            }
        }
    }

#pragma unroll
    for (int k = 0; k < kTierSlots; ++k) {
        const int i = tid + k * kTierThreads;
        if (i >= kTokens) continue;
        const int slot = before[k] + in_group[k];
        tier_out[i] = (uint8_t)tier[k];
        slot_out[i] = (uint16_t)slot;
        const int tier_base = (tier[k] > 0 ? cnt[0] : 0) + (tier[k] > 1 ? cnt[1] : 0) + (tier[k] > 2 ? cnt[2] : 0);
        order_out[tier_base + slot] = (uint16_t)i;
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) res.cnt[t] = cnt[t];
    return res;
}

__device__ __forceinline__ TierCounts tier_rank(TierShared& sh, const TierScores& loaded, const TierParams& tp,
                                                uint8_t* __restrict__ tier_out, uint16_t* __restrict__ slot_out,
                                                uint16_t* __restrict__ order_out) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    TierCounts res = {};

    if (tid == 0) sh.nan_flag = 0;
    float s[kTierSlots];
    uint32_t key[kTierSlots];
    bool has_nan = false;
#pragma unroll
    for (int k = 0; k < kTierSlots; ++k) {
        const int i = tid + k * kTierThreads;
        s[k] = 0.0f;
        key[k] = 0u;
        if (i < kTokens) {
            s[k] = loaded.s[k];
            has_nan |= s[k] != s[k];
            // unsigned key with the same order as the float (and -0 == +0, as the float comparison has it)
            const uint32_t bits = (s[k] == 0.0f) ? 0u : __builtin_bit_cast(uint32_t, s[k]);
            key[k] = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
            reinterpret_cast<uint32_t*>(sh.key4)[i] = key[k];
        }
    }
    __syncthreads();
    if (has_nan) sh.nan_flag = 1;
    __syncthreads();
    if (sh.nan_flag) {
        res.state = 2;
        return res;
    }

    int tier[kTierSlots];
    if (tp.mode == 0) {
        tier_by_thresholds(s, tp.tau_high, tp.tau_med, tp.tau_low, tier);
    } else {
        // rank by (score descending, token index ascending) = number of tokens j with a larger key,
        // or an equal key and j < i.  Work is dealt evenly: tokens 0..511 are two per thread against
        // all 576 keys; the last 64 tokens are taken by all four waves, a quarter of the keys each
        // (partial counts meet in LDS).  All lanes of a wave share the 64-token group of their
        // token, so the comparison regime of a key block is uniform in the wave.
        int rank[kTierSlots];
#pragma unroll
        for (int k = 0; k < 2; ++k) rank[k] = tier_count_above(sh, key[k], tid + k * kTierThreads, 0, kTokens / 4);
        {
            const int wave = tid >> 6;
            const int i = 2 * kTierThreads + lane;                      // 512 + lane, every wave
            const uint32_t me = reinterpret_cast<const uint32_t*>(sh.key4)[i];
            const int part = tier_count_above(sh, me, i, wave * (kTokens / 16), (wave + 1) * (kTokens / 16));
            sh.part_rank[wave][lane] = part;
        }
        if (tid < 3) sh.q[tid] = 0;
        __syncthreads();
        rank[2] = sh.part_rank[0][lane] + sh.part_rank[1][lane] + sh.part_rank[2][lane] + sh.part_rank[3][lane];
        if (tp.mode == 2) {
            // adaptive thresholds: only the quantiles at the target ranks are taken from the ranking
            // (every rank belongs to exactly one token; a rank past the last token leaves 0)
#pragma unroll
            for (int k = 0; k < kTierSlots; ++k) {
                const int i = tid + k * kTierThreads;
                if (i >= kTokens) continue;
                if (rank[k] == tp.k16) sh.q[0] = to_lattice(s[k]);
                if (rank[k] == tp.k16 + tp.k8) sh.q[1] = to_lattice(s[k]);
                if (rank[k] == tp.k16 + tp.k8 + tp.k4) sh.q[2] = to_lattice(s[k]);
            }
            __syncthreads();
            res.state = 3;
#pragma unroll
            for (int j = 0; j < 3; ++j) res.q[j] = sh.q[j];
            return res;
        }
#pragma unroll
        for (int k = 0; k < kTierSlots; ++k) {
            const int i = tid + k * kTierThreads;
            tier[k] = SALI_TIER_PRUNE;
            if (i >= kTokens) continue;
            if (rank[k] < tp.k16 + tp.k8 + tp.k4) tier[k] = SALI_TIER_INT4;
            if (rank[k] < tp.k16 + tp.k8) tier[k] = SALI_TIER_INT8;
            if (rank[k] < tp.k16) tier[k] = SALI_TIER_FP16;
        }
    }
    return tier_finish(sh, tier, tier_out, slot_out, order_out);
}

// Cursor state carried in registers through the frames of one commit pass.
struct CursorRegs {
    int32_t c16, c8, c4, last_src;
    uint32_t faults;
};

// ---- memory budget (Experimental Setup: a strict budget of 784 patches; the eviction rule is this
// library's reading: whole frames leave oldest first until the new frame's kept tokens fit the budget
// and its rows fit the ring-shaped pools) -----------------------------------------------------------
// First row of a run of n rows in a ring pool, -1 if neither candidate place (the cursor, then row 0)
// is free.  The rows of held frames are the window tail .. head, so the test needs no look at the frames.
__device__ __forceinline__ int ring_place(int head, int n, int cap, int tail, int live_rows, int wrapped) {
    if (n == 0) return head;
    if (live_rows == 0) return head + n <= cap ? head : (n <= cap ? 0 : -1);
    if (!wrapped) return head + n <= cap ? head : (n <= tail ? 0 : -1);
    return head + n <= tail ? head : -1;
}

// Budget mode, ONE thread: evicts until the frame fits, then places it.  Returns false if the frame
// cannot be held even by an empty cache.  The ring state is read from and written back to *cur.
__device__ __noinline__ bool tier_place_with_budget(const TierCounts& tc, int frame_id, sali_frame_row* rows,
                                                    CursorRegs& cr, Cursors* cur, int cap16, int cap8, int cap4,
                                                    int budget, int* base_out) {
    RingState rs = cur->ring;
    int head[3] = {cr.c16, cr.c8, cr.c4};
    const int cap[3] = {cap16, cap8, cap4};
    const int n[3] = {tc.cnt[0], tc.cnt[1], tc.cnt[2]};
    const int need = n[0] + n[1] + n[2];
    bool ok;
    for (;;) {
        ok = rs.live_tokens + need <= budget;
        for (int p = 0; p < 3; ++p) {
            base_out[p] = ring_place(head[p], n[p], cap[p], rs.tail[p], rs.live_rows[p], rs.wrapped[p]);
            ok = ok && base_out[p] >= 0;
        }
        if (ok || rs.oldest < 0) break;
        // the oldest held frame leaves
        const int g = rs.oldest;
        const sali_frame_row rg = rows[g];
        const int gb[3] = {rg.base16, rg.base8, rg.base4}, gn[3] = {rg.n16, rg.n8, rg.n4};
        rs.live_tokens -= gn[0] + gn[1] + gn[2];
        for (int p = 0; p < 3; ++p) {
            if (gn[p] == 0) continue;
            rs.live_rows[p] -= gn[p];
            if (rs.live_rows[p] == 0) {
                rs.wrapped[p] = 0;
            } else {
                rs.tail[p] = gb[p] + gn[p];
                if (rs.wrapped[p] && rs.tail[p] == rs.end[p]) {      // the rows before the wrap are all gone
                    rs.tail[p] = 0;
                    rs.wrapped[p] = 0;
                }
            }
        }
        sali_frame_row dead = {};
        dead.frame_id = g;
        dead.src = -1;
        rows[g] = dead;
        // pointer entries behind it hold no data any more; the next stored frame becomes the oldest
        rs.oldest = -1;
        for (int f = g + 1; f < frame_id; ++f) {
            const sali_frame_row r = rows[f];
            if (r.frame_id != f) continue;              // a row that was never written
            if (r.stored) {
                rs.oldest = f;
                break;
            }
            if (r.src == g) rows[f].src = -1;
        }
    }
    if (ok) {
        for (int p = 0; p < 3; ++p) {
            if (n[p] == 0) continue;
            if (rs.live_rows[p] == 0) {
                rs.tail[p] = base_out[p];
                rs.wrapped[p] = 0;
            } else if (!rs.wrapped[p] && base_out[p] == 0) {         // did not fit behind the cursor: wrap
                rs.end[p] = head[p];
                rs.wrapped[p] = 1;
            }
            head[p] = base_out[p] + n[p];
            rs.live_rows[p] += n[p];
        }
        rs.live_tokens += need;
        if (rs.oldest < 0) rs.oldest = frame_id;
        cr.c16 = head[0];
        cr.c8 = head[1];
        cr.c4 = head[2];
    }
    cur->ring = rs;
    return ok;
}

// Frame-table row of one frame from its counts and the running cursors; ONE thread, frames in
// video order.
__device__ __forceinline__ bool tier_commit_one(const TierCounts& tc, int frame_id, sali_frame_row* rows,
                                                CursorRegs& cr, int cap16, int cap8, int cap4, Cursors* cur = nullptr,
                                                int budget = 0, int tiles = 1) {
    sali_frame_row r = {};
    r.frame_id = frame_id;
    if (tc.state == 1) {
        // Algorithm 1: C[t] <- Pointer(C[t-1]); chains resolve to the last stored frame (of a tiled
        // frame: to the last stored entry of the same tile).
        r.src = tiles > 1 ? cur->last_src_tile[frame_id % tiles] : cr.last_src;
        r.stored = 0;
    } else if (tc.state == 2) {
        cr.faults |= SALI_FAULT_NAN_SCORE;
        r.src = -1;
    } else if (budget > 0) {
        int base[3];
        if (tier_place_with_budget(tc, frame_id, rows, cr, cur, cap16, cap8, cap4, budget, base)) {
            r.src = frame_id;
            r.stored = 1;
            r.base16 = base[0];
            r.base8 = base[1];
            r.base4 = base[2];
            r.n16 = tc.cnt[0];
            r.n8 = tc.cnt[1];
            r.n4 = tc.cnt[2];
            r.n_pruned = tc.cnt[3];
            cr.last_src = frame_id;
        } else {
            cr.faults |= SALI_FAULT_OVERFLOW;
            r.src = -1;
        }
    } else if ((long long)cr.c16 + tc.cnt[0] > cap16 || (long long)cr.c8 + tc.cnt[1] > cap8 ||
               (long long)cr.c4 + tc.cnt[2] > cap4) {
        cr.faults |= SALI_FAULT_OVERFLOW;
        r.src = -1;
    } else {
        r.src = frame_id;
        r.stored = 1;
        r.base16 = cr.c16;
        r.base8 = cr.c8;
        r.base4 = cr.c4;
        r.n16 = tc.cnt[0];
        r.n8 = tc.cnt[1];
        r.n4 = tc.cnt[2];
        r.n_pruned = tc.cnt[3];
        cr.c16 += tc.cnt[0];
        cr.c8 += tc.cnt[1];
        cr.c4 += tc.cnt[2];
        cr.last_src = frame_id;
    }
    if (tiles > 1 && r.stored) cur->last_src_tile[frame_id % tiles] = frame_id;
    rows[frame_id] = r;
    return r.stored != 0;
}

// Adaptive thresholds (tier_mode 2; the Discussion says the thresholds need tuning per video domain, the
// Conclusion names adaptive thresholds as future work; the rule is this library's reading): Eq. 8 with the
// thresholds in force; after a stored frame each threshold moves adapt_q8 / 256 of the way to the frame's
// score quantile at its target rank.  Integer arithmetic on the 2^-16 lattice, floor.
// Tiers of one ranked frame (state 3) from the thresholds sh.tau; whole block.
__device__ __forceinline__ TierCounts tier_assign_adaptive(TierShared& sh, const TierScores& loaded,
                                                           uint8_t* __restrict__ tier_out, uint16_t* __restrict__ slot_out,
                                                           uint16_t* __restrict__ order_out) {
    int tier[kTierSlots];
    const float th = (float)sh.tau[0] * (1.0f / 65536.0f), tm = (float)sh.tau[1] * (1.0f / 65536.0f),
                tl = (float)sh.tau[2] * (1.0f / 65536.0f);          // exact: at most 17 significant bits
    tier_by_thresholds(loaded.s, th, tm, tl, tier);
    return tier_finish(sh, tier, tier_out, slot_out, order_out);
}

// ONE thread, after the frame's row is written
__device__ __forceinline__ void tier_adapt_update(TierShared& sh, const int* q, int adapt_q8) {
#pragma unroll
    for (int j = 0; j < 3; ++j) sh.tau[j] += ((q[j] - sh.tau[j]) * adapt_q8) >> 8;      // arithmetic shift = floor
}

__device__ __forceinline__ CursorRegs cursor_load(const Cursors* cur) {
    CursorRegs cr;
    cr.c16 = cur->c16;
    cr.c8 = cur->c8;
    cr.c4 = cur->c4;
    cr.last_src = cur->last_src;
    cr.faults = 0u;
    return cr;
}

__device__ __forceinline__ void cursor_store(Cursors* cur, const CursorRegs& cr) {
    cur->c16 = cr.c16;
    cur->c8 = cr.c8;
    cur->c4 = cr.c4;
    cur->last_src = cr.last_src;
    if (cr.faults != 0u) atomicOr(&cur->status, cr.faults);
}

// both parts for one frame (whole block)
__device__ __forceinline__ void tier_body(TierShared& sh, const float* scores, bool redundant, const TierParams& tp,
                                          int frame_id, sali_frame_row* rows, uint8_t* __restrict__ tier_out,
                                          uint16_t* __restrict__ slot_out, uint16_t* __restrict__ order_out,
                                          Cursors* cur, int cap16, int cap8, int cap4, int budget, int tiles) {
    TierCounts tc = {};
    tc.state = 1;
    const TierScores loaded = tier_load_scores(scores);
    if (!redundant) tc = tier_rank(sh, loaded, tp, tier_out, slot_out, order_out);
    int q[3] = {tc.q[0], tc.q[1], tc.q[2]};
    const bool adaptive = tc.state == 3;
    if (adaptive) {
        if (threadIdx.x < 3) sh.tau[threadIdx.x] = cur->adapt_tau[threadIdx.x];
        __syncthreads();
        tc = tier_assign_adaptive(sh, loaded, tier_out, slot_out, order_out);
    }
    if (threadIdx.x == 0) {
        CursorRegs cr = cursor_load(cur);
        const bool stored = tier_commit_one(tc, frame_id, rows, cr, cap16, cap8, cap4, cur, budget, tiles);
        cursor_store(cur, cr);
        if (adaptive && stored) {
            tier_adapt_update(sh, q, tp.adapt_q8);
#pragma unroll
            for (int j = 0; j < 3; ++j) cur->adapt_tau[j] = sh.tau[j];
        }
    }
}

}  // namespace sali
