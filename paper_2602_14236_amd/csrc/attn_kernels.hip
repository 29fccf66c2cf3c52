// Single-query attention that reads the mixed-precision pools directly (gfx950).
//
// Just-In-Time Dequantization (entries are dequantised while attention is computed) and
// Implementation Details (the dequantisation is fused with the attention computation).  For one
// layer and every head h: s_j = softmax_scale * <q_h, K^_j>, out_h = softmax(s) V^, over the logical
// token sequence of a frame range.  K^, V^ are the dequantise-on-read values (fp16-rounded, exactly
// what k_unpack writes); a redundant frame's entry is a pointer (Algorithm 1), so its source
// frame's tokens count once more; pruned tokens are not in the cache.
//
// One query per head makes Q K^T and P V matrix-vector products: 2 flops per byte read, so the
// kernel is bound by HBM and written as a stream, not for MFMA.  The compressed rows are read
// once, in pool order (attention does not care about token order), with the same lane mapping as
// the pack / unpack kernels: a row is handled by 16 adjacent lanes holding 8 consecutive head-dim
// values each, a 32-value quantisation group is one lane quad, the dot product is reduced over the
// 16 lanes with four DPP moves.  Every lane group keeps an online-softmax state (running max, sum
// and 8 output values per lane); a block merges its 16 lane groups through LDS and writes one
// partial (max, sum, 128 values); a second small kernel merges the partials of a head.
//
// This file must be compiled with -ffp-contract=off: the dequantised values must be bit-identical
// to those of the unpack kernel (one fp32 multiply or fused multiply-add, then fp16 rounding).

#include "sali_internal.h"

namespace sali {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kRowsPerStep = 4;               // rows in flight per lane group (K and V each)
constexpr int kPartialStride = kHeadDim + 2;  // max, sum, 128 values

union Row16B {
    u32x4 u;
    _Float16 h[8];
};

// see kv_kernels.hip: keeps the fp32 product and the fp16 rounding two separate roundings
__device__ __forceinline__ float round_to_half(float v) {
    asm volatile("" : "+v"(v));
    return (float)(_Float16)v;
}

template <int kCtrl>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, true));
}

// sum over the 16 lanes of a row: lane ^ 1, lane ^ 2 inside the quad, then mirror inside 8 and
// inside 16 lanes (every lane ends with the full sum)
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_move<0xB1>(v);       // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);       // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);      // row_half_mirror
    v += dpp_move<0x140>(v);      // row_mirror
    return v;
}

// raw 16-byte (or shorter) piece of one pool row for one lane, plus its group's scale / zero
struct RawRow {
    u32x4 u;
    float scale, zero;
    int tier;                     // SALI_TIER_*, SALI_TIER_PRUNE = nothing to read
};

__device__ __forceinline__ RawRow load_row(const Pools& pools, size_t plane, const sali_frame_row& row, int j, int l) {
    RawRow r;
    r.u = (u32x4){0u, 0u, 0u, 0u};
    r.scale = 0.0f;
    r.zero = 0.0f;
    r.tier = SALI_TIER_PRUNE;
    const int n16 = row.n16, n8 = row.n8, n4 = row.n4;
    if (j < n16) {
        r.tier = SALI_TIER_FP16;
        const u32x4* p = reinterpret_cast<const u32x4*>(pools.p16) + ((plane * pools.cap16 + row.base16 + j) * 16 + l);
        r.u = __builtin_nontemporal_load(p);
    } else if (j < n16 + n8) {
        r.tier = SALI_TIER_INT8;
        const size_t prow = plane * pools.cap8 + row.base8 + (j - n16);
        const u32x2* p = reinterpret_cast<const u32x2*>(pools.c8 + prow * kHeadDim) + l;
        const u32x2 c = __builtin_nontemporal_load(p);
        r.u.x = c.x;
        r.u.y = c.y;
        r.scale = pools.s8[prow * kGroupsPerRow + (l >> 2)];
    } else if (j < n16 + n8 + n4) {
        r.tier = SALI_TIER_INT4;
        const size_t prow = plane * pools.cap4 + row.base4 + (j - n16 - n8);
        const uint32_t* p = reinterpret_cast<const uint32_t*>(pools.c4 + prow * (kHeadDim / 2)) + l;
        r.u.x = __builtin_nontemporal_load(p);
        r.scale = pools.s4[prow * kGroupsPerRow + (l >> 2)];
        r.zero = (float)__builtin_bit_cast(_Float16, pools.z4[prow * kGroupsPerRow + (l >> 2)]);
    }
    return r;
}

// the lane's 8 dequantise-on-read values of a row (the arithmetic of k_unpack)
__device__ __forceinline__ void dequant_row(const RawRow& r, float x[8]) {
    if (r.tier == SALI_TIER_FP16) {
        Row16B v;
        v.u = r.u;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (float)v.h[e];
    } else if (r.tier == SALI_TIER_INT8) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t word = e < 4 ? r.u.x : r.u.y;
            const int q = (int)(int8_t)((word >> (8 * (e & 3))) & 0xFF);
            x[e] = round_to_half((float)q * r.scale);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int q = (int)((r.u.x >> (4 * e)) & 0xF);
            x[e] = round_to_half(__builtin_fmaf((float)q, r.scale, r.zero));
        }
    }
}

}  // namespace

// grid (n_chunks * n_splits, n_heads).  Block (c, s) of head h takes the frames
// [frame_lo + c * frames_per_chunk, ...) and of each source frame the 64-row groups s, s + n_splits, ...
__global__ __launch_bounds__(256) void k_attn_partial(const sali_frame_row* __restrict__ rows, Pools pools, int layer,
                                                      int n_heads, const _Float16* __restrict__ q, int frame_lo,
                                                      int frame_hi, int frames_per_chunk, int n_splits,
                                                      float softmax_scale, float* __restrict__ partial) {
    __shared__ float s_m[16], s_l[16];
    __shared__ float s_acc[16][kHeadDim];
    __shared__ int s_src, s_mult;

    const int h = blockIdx.y;
    const int chunk = blockIdx.x / n_splits, split = blockIdx.x % n_splits;
    const int g = threadIdx.x >> 4, l = threadIdx.x & 15;
    const size_t plane_k = ((size_t)layer * 2 + 0) * n_heads + h;
    const size_t plane_v = ((size_t)layer * 2 + 1) * n_heads + h;

    float qf[8];
    {
        Row16B qv;
        qv.u = reinterpret_cast<const u32x4*>(q)[h * 16 + l];
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[e] = (float)qv.h[e];
    }

    float mx = -INFINITY, lsum = 0.0f;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;

    const int f0 = frame_lo + chunk * frames_per_chunk;
    const int f1 = min(frame_hi, f0 + frames_per_chunk);
    for (int f = f0; f < f1; ++f) {
        // Which stored frame does frame f bring in, and how many times?  A stored frame counts for
        // itself and for the redundant frames behind it (up to the next stored frame or the end of
        // the range); redundant frames at the head of the range, whose source lies before it, are
        // counted at the first of them.  One thread decides, the block follows.
        if (threadIdx.x == 0) {
            int src = -1, mult = 0;
            const sali_frame_row r = rows[f];
            bool leader = false;
            if (r.stored != 0) {
                leader = true;
            } else if (r.src >= 0 && r.src < frame_lo) {
                leader = true;
                for (int t = frame_lo; t < f; ++t)
                    if (rows[t].src == r.src) leader = false;      // an earlier frame of the run counts them
            }
            if (leader) {
                src = r.src;
                mult = 1;
                for (int t = f + 1; t < frame_hi && rows[t].stored == 0; ++t)
                    if (rows[t].src == src) ++mult;
            }
            s_src = src;
            s_mult = mult;
        }
        __syncthreads();
        const int src = s_src;
        const float mult = (float)s_mult;
        __syncthreads();
        if (src < 0) continue;
        const sali_frame_row row = rows[src];
        const int nkeep = row.n16 + row.n8 + row.n4;

        for (int jb = split * 64; jb < nkeep; jb += n_splits * 64) {
            RawRow rk[kRowsPerStep], rv[kRowsPerStep];
#pragma unroll
            for (int r = 0; r < kRowsPerStep; ++r) {
                const int j = jb + r * 16 + g;
                rk[r] = load_row(pools, plane_k, row, j, l);
                rv[r] = load_row(pools, plane_v, row, j, l);
            }
            float s[kRowsPerStep];
            float bm = -INFINITY;
#pragma unroll
            for (int r = 0; r < kRowsPerStep; ++r) {
                float x[8];
                dequant_row(rk[r], x);
                float d = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d += qf[e] * x[e];
                d = row16_sum(d);
                s[r] = rk[r].tier == SALI_TIER_PRUNE ? -INFINITY : softmax_scale * d;
                bm = fmaxf(bm, s[r]);
            }
            const float new_mx = fmaxf(mx, bm);
            if (new_mx == -INFINITY) continue;          // nothing seen yet (uniform inside the lane group)
            const float corr = expf(mx - new_mx);       // mx = -inf: 0
            lsum *= corr;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] *= corr;
#pragma unroll
            for (int r = 0; r < kRowsPerStep; ++r) {
                const float p = mult * expf(s[r] - new_mx);     // absent row: exp(-inf) = 0
                float x[8];
                dequant_row(rv[r], x);
                lsum += p;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += p * x[e];
            }
            mx = new_mx;
        }
    }

    // merge the 16 lane groups
    if (l == 0) {
        s_m[g] = mx;
        s_l[g] = lsum;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_acc[g][8 * l + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < kHeadDim) {
        float big = -INFINITY;
#pragma unroll
        for (int k = 0; k < 16; ++k) big = fmaxf(big, s_m[k]);
        float lt = 0.0f, at = 0.0f;
        if (big != -INFINITY) {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const float w = expf(s_m[k] - big);
                lt += w * s_l[k];
                at += w * s_acc[k][threadIdx.x];
            }
        }
        float* out = partial + ((size_t)h * kAttnPartials + blockIdx.x) * kPartialStride;
        if (threadIdx.x == 0) {
            out[0] = big;
            out[1] = lt;
        }
        out[2 + threadIdx.x] = at;
    }
}

// grid (n_heads), 128 threads: merge of the head's partials
__global__ __launch_bounds__(kHeadDim) void k_attn_merge(const float* __restrict__ partial, int n_partials,
                                                         float* __restrict__ out, float* __restrict__ lse) {
    const int h = blockIdx.x;
    const float* p = partial + (size_t)h * kAttnPartials * kPartialStride;
    float big = -INFINITY;
    for (int k = 0; k < n_partials; ++k) big = fmaxf(big, p[(size_t)k * kPartialStride]);
    float lt = 0.0f, at = 0.0f;
    if (big != -INFINITY) {
        for (int k = 0; k < n_partials; ++k) {
            const float w = expf(p[(size_t)k * kPartialStride] - big);
            lt += w * p[(size_t)k * kPartialStride + 1];
            at += w * p[(size_t)k * kPartialStride + 2 + threadIdx.x];
        }
    }
    out[h * kHeadDim + threadIdx.x] = lt > 0.0f ? at / lt : 0.0f;
    if (lse != nullptr && threadIdx.x == 0) lse[h] = lt > 0.0f ? big + logf(lt) : -INFINITY;
}

hipError_t launch_attend(const sali_frame_row* d_rows, Pools pools, int layer, int n_heads, const void* d_q,
                         int frame_lo, int frame_hi, float softmax_scale, float* d_partial, float* d_out,
                         float* d_lse_or_null, hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t s) {
    const int n_range = frame_hi - frame_lo;
    int n_partials = 0;
    if (n_range > 0) {
        const int fpc = (n_range + kAttnPartials - 1) / kAttnPartials;
        const int n_chunks = (n_range + fpc - 1) / fpc;
        // short ranges: split every frame's rows over several blocks (576 rows = 9 groups of 64)
        int n_splits = (2048 + n_chunks * n_heads - 1) / (n_chunks * n_heads);
        n_splits = n_splits < 1 ? 1 : (n_splits > 9 ? 9 : n_splits);
        if (n_splits > kAttnPartials / n_chunks) n_splits = kAttnPartials / n_chunks;
        n_partials = n_chunks * n_splits;
        if (ev_start != nullptr && hipEventRecord(ev_start, s) != hipSuccess) return hipErrorUnknown;
        hipLaunchKernelGGL(k_attn_partial, dim3(n_partials, n_heads), dim3(256), 0, s, d_rows, pools, layer, n_heads,
                           reinterpret_cast<const _Float16*>(d_q), frame_lo, frame_hi, fpc, n_splits, softmax_scale,
                           d_partial);
        if (ev_stop != nullptr && hipEventRecord(ev_stop, s) != hipSuccess) return hipErrorUnknown;
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_attn_merge, dim3(n_heads), dim3(kHeadDim), 0, s, d_partial, n_partials, d_out, d_lse_or_null);
    return hipGetLastError();
}

}  // namespace sali
