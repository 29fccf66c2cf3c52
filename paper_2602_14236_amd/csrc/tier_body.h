// Tier assignment (Eq. 8 or top-k counts), compaction indices and frame-table row for one frame.
// Shared by the stand-alone tier kernel and by the last block of the pooling kernel; must be
// entered by a whole block of exactly 576 threads, one per token.  Only comparisons and integer
// arithmetic: the result does not depend on floating-point contraction settings.
#pragma once

#include "sali_internal.h"

namespace sali {

struct TierShared {
    uint4 key4[kTokens / 4];        // order-preserving integer image of the scores
    int wave_cnt[kTokens / 64][4];
    int nan_flag;
};

__device__ __forceinline__ void tier_body(TierShared& sh, const float* scores, bool redundant, const TierParams& tp,
                                          int frame_id, sali_frame_row* rows, uint8_t* __restrict__ tier_out,
                                          uint16_t* __restrict__ slot_out, uint16_t* __restrict__ order_out,
                                          Cursors* cur, int cap16, int cap8, int cap4) {
    const int i = threadIdx.x;
    const int wave = i >> 6, lane = i & 63;

    if (redundant) {
        // Algorithm 1: C[t] <- Pointer(C[t-1]); chains resolve to the last stored frame.
        if (i == 0) {
            sali_frame_row r = {};
            r.frame_id = frame_id;
            r.src = cur->last_src;
            r.stored = 0;
            rows[frame_id] = r;
        }
        return;
    }

    const float s = __hip_atomic_load(scores + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // unsigned key with the same order as the float (and -0 == +0, as the float comparison has it)
    uint32_t bits = (s == 0.0f) ? 0u : __builtin_bit_cast(uint32_t, s);
    const uint32_t key = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
    reinterpret_cast<uint32_t*>(sh.key4)[i] = key;
    if (i == 0) sh.nan_flag = 0;
    __syncthreads();
    if (s != s) sh.nan_flag = 1;
    __syncthreads();
    if (sh.nan_flag) {
        if (i == 0) {
            atomicOr(&cur->status, SALI_FAULT_NAN_SCORE);
            sali_frame_row r = {};
            r.frame_id = frame_id;
            r.src = -1;
            rows[frame_id] = r;
        }
        return;
    }

    int tier;
    if (tp.mode == 0) {
        // Eq. 8, inequalities as printed
        tier = SALI_TIER_PRUNE;
        if (s > tp.tau_low) tier = SALI_TIER_INT4;
        if (s > tp.tau_med) tier = SALI_TIER_INT8;
        if (s > tp.tau_high) tier = SALI_TIER_FP16;
    } else {
        // rank by (score descending, token index ascending) = number of tokens j with a larger key,
        // or an equal key and j < i.  Tokens of earlier waves count with >=, of later waves with >,
        // so only the 64 tokens of the own wave need the index test.  128-bit broadcast LDS reads.
        int rank = 0;
        const int own0 = wave * 16, own1 = own0 + 16;
#pragma unroll 4
        for (int j4 = 0; j4 < own0; ++j4) {
            const uint4 v = sh.key4[j4];
            rank += (v.x >= key ? 1 : 0) + (v.y >= key ? 1 : 0) + (v.z >= key ? 1 : 0) + (v.w >= key ? 1 : 0);
        }
#pragma unroll 4
        for (int j4 = own0; j4 < own1; ++j4) {
            const uint4 v = sh.key4[j4];
            const int j = 4 * j4;
            rank += (v.x > key || (v.x == key && j < i)) ? 1 : 0;
            rank += (v.y > key || (v.y == key && j + 1 < i)) ? 1 : 0;
            rank += (v.z > key || (v.z == key && j + 2 < i)) ? 1 : 0;
            rank += (v.w > key || (v.w == key && j + 3 < i)) ? 1 : 0;
        }
#pragma unroll 4
        for (int j4 = own1; j4 < kTokens / 4; ++j4) {
            const uint4 v = sh.key4[j4];
            rank += (v.x > key ? 1 : 0) + (v.y > key ? 1 : 0) + (v.z > key ? 1 : 0) + (v.w > key ? 1 : 0);
        }
        tier = SALI_TIER_PRUNE;
        if (rank < tp.k16 + tp.k8 + tp.k4) tier = SALI_TIER_INT4;
        if (rank < tp.k16 + tp.k8) tier = SALI_TIER_INT8;
        if (rank < tp.k16) tier = SALI_TIER_FP16;
    }

    // slot = number of earlier tokens in the same tier (ballot inside the wave + wave prefix)
    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int in_wave = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const unsigned long long m = __ballot(tier == k);
        if (tier == k) in_wave = __popcll(m & lt_mask);
        if (lane == 0) sh.wave_cnt[wave][k] = __popcll(m);
    }
    __syncthreads();
    int before = 0;
    int cnt[4] = {0, 0, 0, 0};
    for (int w = 0; w < kTokens / 64; ++w) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = sh.wave_cnt[w][k];
            cnt[k] += c;
            if (w < wave && k == tier) before += c;
        }
    }
    const int slot = before + in_wave;

    // capacity check (uniform: every thread reads the same cursors)
    const int c16 = cur->c16, c8 = cur->c8, c4 = cur->c4;
    const bool overflow = (long long)c16 + cnt[0] > cap16 || (long long)c8 + cnt[1] > cap8 ||
                          (long long)c4 + cnt[2] > cap4;
    __syncthreads();    // all cursor reads precede the update below
    if (overflow) {
        if (i == 0) {
            atomicOr(&cur->status, SALI_FAULT_OVERFLOW);
            sali_frame_row r = {};
            r.frame_id = frame_id;
            r.src = -1;
            rows[frame_id] = r;
        }
        return;
    }

    tier_out[i] = (uint8_t)tier;
    slot_out[i] = (uint16_t)slot;
    const int tier_base = (tier > 0 ? cnt[0] : 0) + (tier > 1 ? cnt[1] : 0) + (tier > 2 ? cnt[2] : 0);
    order_out[tier_base + slot] = (uint16_t)i;

    if (i == 0) {
        sali_frame_row r = {};
        r.frame_id = frame_id;
        r.src = frame_id;
        r.stored = 1;
        r.base16 = c16;
        r.base8 = c8;
        r.base4 = c4;
        r.n16 = cnt[0];
        r.n8 = cnt[1];
        r.n4 = cnt[2];
        r.n_pruned = cnt[3];
        rows[frame_id] = r;
        cur->c16 = c16 + cnt[0];
        cur->c8 = c8 + cnt[1];
        cur->c4 = c4 + cnt[2];
        cur->last_src = frame_id;
    }
}

}  // namespace sali
