// Tier assignment, compaction indices, mixed-precision K/V pack and unpack for gfx950.
//
// Spatial Filtering via Saliency-Guided Quantization (Eq. 8), Algorithm 1 ("Store (K_i, V_i)
// with precision Q(s_i)"), Implementation Details (symmetric min-max INT8, asymmetric INT4)
// and Just-In-Time Dequantization.
//
// This file must be compiled with -ffp-contract=off: every quantisation step is one IEEE
// fp32 operation (divide, multiply, subtract, round-half-even) and the only fused
// multiply-add is the one written out in the INT4 dequantiser.
//
// Data movement: a K/V row (one token in one layer / K|V / head) is 128 halves = 256 B and is
// handled by 16 adjacent lanes, 16 B each, so a wave moves four rows per instruction and a
// 32-value quantisation group sits in one lane quad (reductions are two DPP quad swaps).
// Rows are visited in pool order (all FP16 tokens, then INT8, then INT4, in token order inside
// a tier), so pool writes are contiguous runs and pruned tokens are never read.

#include "sali_internal.h"
#include "tier_body.h"

namespace sali {

namespace {

constexpr int kRowsPerBlock = 64;      // 16 lane-groups x 4 rows
constexpr int kRowsPerLaneGroup = 4;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

union Row16B {
    u32x4 u;
    _Float16 h[8];
    uint16_t s[8];
};

__device__ __forceinline__ u32x4 zero4() { return (u32x4){0u, 0u, 0u, 0u}; }

__device__ __forceinline__ float quad_swap1(float v) {      // lane ^ 1 inside a quad
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float quad_swap2(float v) {      // lane ^ 2 inside a quad
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
}
// fp32 -> fp16 (nearest even) of a value that must first exist as a rounded fp32 number.  The
// empty asm keeps the compiler from merging the producing fp32 operation and the conversion
// into one mixed-precision instruction, which would round the exact result once instead of twice.
__device__ __forceinline__ _Float16 to_half_after_f32(float v) {
    asm volatile("" : "+v"(v));
    return (_Float16)v;
}

__device__ __forceinline__ float quad_max(float v) {
    v = fmaxf(v, quad_swap1(v));
    return fmaxf(v, quad_swap2(v));
}
__device__ __forceinline__ float quad_min(float v) {
    v = fminf(v, quad_swap1(v));
    return fminf(v, quad_swap2(v));
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Tier + rank + compaction indices: one block of 256 threads (see tier_body.h).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kTierThreads) void k_tier(const float* __restrict__ scores, const sali_gate* gate,
                                                  TierParams tp, int frame_id, sali_frame_row* rows,
                                                  uint8_t* __restrict__ tier_out, uint16_t* __restrict__ slot_out,
                                                  uint16_t* __restrict__ order_out, Cursors* cur, int cap16,
                                                  int cap8, int cap4) {
    __shared__ TierShared sh;
    const bool redundant = gate != nullptr && gate->redundant != 0;
    tier_body(sh, scores, redundant, tp, frame_id, rows, tier_out, slot_out, order_out, cur, cap16, cap8, cap4);
}

// ---------------------------------------------------------------------------------------------
// Pack: grid (ceil(576 / 64), planes, frames); plane = (layer, K|V, head); frame i of the launch has
// id first_frame_id + i.
// ---------------------------------------------------------------------------------------------
// kNTL / kNTS: non-temporal loads / stores
template <bool kNTL, bool kNTS>
__global__ __launch_bounds__(256) void k_pack(KvBatch f, const sali_frame_row* __restrict__ rows, int first_frame_id,
                                              const uint16_t* __restrict__ order_base, Pools pools, Cursors* cur) {
    const int frame_id = first_frame_id + (int)blockIdx.z;
    const u32x4* __restrict__ kv = reinterpret_cast<const u32x4*>(f.kv[blockIdx.z]);
    const uint16_t* __restrict__ order = order_base + (size_t)frame_id * kTokens;
    const sali_frame_row row = rows[frame_id];
    if (row.stored == 0) return;
    const int n16 = row.n16, n8 = row.n8;
    const int nkeep = n16 + n8 + row.n4;
    const int j0 = blockIdx.x * kRowsPerBlock;
    if (j0 >= nkeep) return;
    const size_t plane = blockIdx.y;
    const int g = threadIdx.x >> 4;     // lane group = one row per step
    const int l = threadIdx.x & 15;     // 16-byte chunk of the row

    Row16B v[kRowsPerLaneGroup];
    int jj[kRowsPerLaneGroup];
#pragma unroll
    for (int r = 0; r < kRowsPerLaneGroup; ++r) {
        const int j = j0 + r * 16 + g;
        jj[r] = j;
        if (j < nkeep) {
            const int tok = order[j];
            v[r].u = kNTL ? __builtin_nontemporal_load(&kv[(plane * kTokens + tok) * 16 + l]) : kv[(plane * kTokens + tok) * 16 + l];
        } else {
            v[r].u = zero4();
        }
    }

    bool bad = false;
#pragma unroll
    for (int r = 0; r < kRowsPerLaneGroup; ++r) {
        const int j = jj[r];
        if (j >= nkeep) continue;
        if (j < n16) {
            // FP16 tier: verbatim copy
#pragma unroll
            for (int e = 0; e < 8; ++e) bad |= (v[r].s[e] & 0x7C00u) == 0x7C00u;
            u32x4* dst = reinterpret_cast<u32x4*>(pools.p16) + ((plane * pools.cap16 + row.base16 + j) * 16 + l);
            if (kNTS) __builtin_nontemporal_store(v[r].u, dst); else *dst = v[r].u;
        } else if (j < n16 + n8) {
            // INT8, symmetric: scale = max|x| / 127, q = rne(x * (127 / max|x|))
            float x[8];
            float m = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[e] = (float)v[r].h[e];
                m = fmaxf(m, fabsf(x[e]));
                bad |= (v[r].s[e] & 0x7C00u) == 0x7C00u;
            }
            m = quad_max(m);
            const bool nz = m > 0.0f;
            const float scale = nz ? m / 127.0f : 0.0f;
            const float inv = nz ? 127.0f / m : 0.0f;
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int q = (int)rintf(x[e] * inv);
                q = min(127, max(-127, q));
                if (e < 4) lo |= (uint32_t)(q & 0xFF) << (8 * e);
                else hi |= (uint32_t)(q & 0xFF) << (8 * (e - 4));
            }
            const size_t prow = plane * pools.cap8 + row.base8 + (j - n16);
            u32x2* dst = reinterpret_cast<u32x2*>(pools.c8 + prow * kHeadDim) + l;
            if (kNTS) __builtin_nontemporal_store((u32x2){lo, hi}, dst); else *dst = (u32x2){lo, hi};
            if ((l & 3) == 0) pools.s8[prow * kGroupsPerRow + (l >> 2)] = scale;
        } else {
            // INT4, asymmetric: scale = (max - min) / 15, q = rne((x - min) * (15 / (max - min)))
            float x[8];
            float mn = (float)v[r].h[0], mx = mn;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[e] = (float)v[r].h[e];
                mn = fminf(mn, x[e]);
                mx = fmaxf(mx, x[e]);
                bad |= (v[r].s[e] & 0x7C00u) == 0x7C00u;
            }
            mn = quad_min(mn);
            mx = quad_max(mx);
            const float range = mx - mn;
            const bool nz = range > 0.0f;
            const float scale = nz ? range / 15.0f : 0.0f;
            const float inv = nz ? 15.0f / range : 0.0f;
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = x[e] - mn;
                int q = (int)rintf(d * inv);
                q = min(15, max(0, q));
                packed |= (uint32_t)q << (4 * e);       // element 2k low nibble, 2k+1 high nibble of byte k
            }
            const size_t prow = plane * pools.cap4 + row.base4 + (j - n16 - n8);
            uint32_t* dst = reinterpret_cast<uint32_t*>(pools.c4 + prow * (kHeadDim / 2)) + l;
            if (kNTS) __builtin_nontemporal_store(packed, dst); else *dst = packed;
            if ((l & 3) == 0) {
                pools.s4[prow * kGroupsPerRow + (l >> 2)] = scale;
                pools.z4[prow * kGroupsPerRow + (l >> 2)] = __builtin_bit_cast(uint16_t, (_Float16)mn);
            }
        }
    }
    if (bad) atomicOr(&cur->status, SALI_FAULT_NONFINITE);
}

// ---------------------------------------------------------------------------------------------
// Unpack: grid (576 / 64, planes, frames); rebuilds the dense fp16 frames in token order; frame i of
// the launch has id first_frame_id + i and its validity mask at valid_base + i * 576.
// ---------------------------------------------------------------------------------------------
template <bool kNTL, bool kNTS>
__global__ __launch_bounds__(256) void k_unpack(const sali_frame_row* __restrict__ rows, int first_frame_id,
                                                const uint16_t* __restrict__ order_base, Pools pools, KvBatch f,
                                                uint8_t* valid_base, Cursors* cur) {
    const int frame_id = first_frame_id + (int)blockIdx.z;
    u32x4* __restrict__ out = reinterpret_cast<u32x4*>(f.kv[blockIdx.z]);
    uint8_t* valid = valid_base != nullptr ? valid_base + (size_t)blockIdx.z * kTokens : nullptr;
    const int src = rows[frame_id].src;
    const size_t plane = blockIdx.y;
    const int g = threadIdx.x >> 4;
    const int l = threadIdx.x & 15;
    const int j0 = blockIdx.x * kRowsPerBlock;
    if (src < 0) {
        // nothing stored under this id: read back as an all-pruned frame
#pragma unroll
        for (int r = 0; r < kRowsPerLaneGroup; ++r) {
            const int tok = j0 + r * 16 + g;
            out[(plane * kTokens + tok) * 16 + l] = zero4();
            if (valid != nullptr && plane == 0 && l == 0) valid[tok] = 0;
        }
        if (blockIdx.x == 0 && plane == 0 && threadIdx.x == 0) atomicOr(&cur->status, SALI_FAULT_NO_DATA);
        return;
    }
    const sali_frame_row row = rows[src];
    const uint16_t* order = order_base + (size_t)src * kTokens;
    const int n16 = row.n16, n8 = row.n8, n4 = row.n4;

    int tok[kRowsPerLaneGroup];
    Row16B raw[kRowsPerLaneGroup];
    float scale[kRowsPerLaneGroup], zero[kRowsPerLaneGroup];
#pragma unroll
    for (int r = 0; r < kRowsPerLaneGroup; ++r) {
        const int j = j0 + r * 16 + g;          // always < 576
        tok[r] = order[j];
        raw[r].u = zero4();
        scale[r] = 0.0f;
        zero[r] = 0.0f;
        if (j < n16) {
            const u32x4* srcp = reinterpret_cast<const u32x4*>(pools.p16) + ((plane * pools.cap16 + row.base16 + j) * 16 + l);
            raw[r].u = kNTL ? __builtin_nontemporal_load(srcp) : *srcp;
        } else if (j < n16 + n8) {
            const size_t prow = plane * pools.cap8 + row.base8 + (j - n16);
            const u32x2* srcp = reinterpret_cast<const u32x2*>(pools.c8 + prow * kHeadDim) + l;
            const u32x2 c = kNTL ? __builtin_nontemporal_load(srcp) : *srcp;
            raw[r].u.x = c.x;
            raw[r].u.y = c.y;
            scale[r] = pools.s8[prow * kGroupsPerRow + (l >> 2)];
        } else if (j < n16 + n8 + n4) {
            const size_t prow = plane * pools.cap4 + row.base4 + (j - n16 - n8);
            const uint32_t* srcp = reinterpret_cast<const uint32_t*>(pools.c4 + prow * (kHeadDim / 2)) + l;
            raw[r].u.x = kNTL ? __builtin_nontemporal_load(srcp) : *srcp;
            scale[r] = pools.s4[prow * kGroupsPerRow + (l >> 2)];
            zero[r] = (float)__builtin_bit_cast(_Float16, pools.z4[prow * kGroupsPerRow + (l >> 2)]);
        }
    }
#pragma unroll
    for (int r = 0; r < kRowsPerLaneGroup; ++r) {
        const int j = j0 + r * 16 + g;
        Row16B o;
        if (j < n16) {
            o.u = raw[r].u;
        } else if (j < n16 + n8) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t word = e < 4 ? raw[r].u.x : raw[r].u.y;
                const int q = (int)(int8_t)((word >> (8 * (e & 3))) & 0xFF);
                o.h[e] = to_half_after_f32((float)q * scale[r]);          // one fp32 multiply, then RNE to fp16
            }
        } else if (j < n16 + n8 + n4) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int q = (int)((raw[r].u.x >> (4 * e)) & 0xF);
                o.h[e] = to_half_after_f32(__builtin_fmaf((float)q, scale[r], zero[r]));   // fused: one fp32 rounding
            }
        } else {
            o.u = zero4();
        }
        if (kNTS) __builtin_nontemporal_store(o.u, &out[(plane * kTokens + tok[r]) * 16 + l]);
        else out[(plane * kTokens + tok[r]) * 16 + l] = o.u;
        if (valid != nullptr && plane == 0 && l == 0) valid[tok[r]] = (j < n16 + n8 + n4) ? 1 : 0;
    }
}

// ---------------------------------------------------------------------------------------------
hipError_t launch_tier(const float* d_scores, const sali_gate* d_gate_or_null, TierParams tp, int frame_id,
                       sali_frame_row* d_rows, uint8_t* d_tier, uint16_t* d_slot, uint16_t* d_order,
                       Cursors* d_cur, Pools pools, hipStream_t s) {
    hipLaunchKernelGGL(k_tier, dim3(1), dim3(kTierThreads), 0, s, d_scores, d_gate_or_null, tp, frame_id, d_rows,
                       d_tier, d_slot, d_order, d_cur, pools.cap16, pools.cap8, pools.cap4);
    return hipGetLastError();
}

hipError_t launch_pack(const KvBatch& f, int n, const sali_frame_row* d_rows, int first_frame_id,
                       const uint16_t* d_order_base, Pools pools, Cursors* d_cur, int n_planes, hipStream_t s) {
    dim3 grid((kTokens + kRowsPerBlock - 1) / kRowsPerBlock, n_planes, n);
    // streaming both ways: non-temporal loads and stores.  (Ordinary stores keep the new pool rows in
    // the last-level cache, which speeds up an immediate read-back by about as much as it slows this
    // kernel; without an immediate read-back non-temporal stores measured 10 % faster.)
    hipLaunchKernelGGL((k_pack<true, true>), grid, dim3(256), 0, s, f, d_rows, first_frame_id, d_order_base, pools,
                       d_cur);
    return hipGetLastError();
}

hipError_t launch_unpack(const sali_frame_row* d_rows, int first_frame_id, const uint16_t* d_order_base, Pools pools,
                         const KvBatch& out, int n, uint8_t* d_valid_or_null, Cursors* d_cur, int n_planes,
                         hipStream_t s) {
    dim3 grid(kTokens / kRowsPerBlock, n_planes, n);
    hipLaunchKernelGGL((k_unpack<true, true>), grid, dim3(256), 0, s, d_rows, first_frame_id, d_order_base, pools, out,
                       d_valid_or_null, d_cur);
    return hipGetLastError();
}

}  // namespace sali
