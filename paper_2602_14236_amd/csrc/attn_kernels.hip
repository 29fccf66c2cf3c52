// Single-query attention that reads the mixed-precision pools directly (gfx950).
//
// Just-In-Time Dequantization (entries are dequantised while attention is computed) and
// Implementation Details (the dequantisation is fused with the attention computation).  For one
// layer and every head h: s_j = softmax_scale * <q_h, K^_j>, out_h = softmax(s) V^, over the logical
// token sequence of a frame range.  "Fused" is taken literally: the dequantised values
// K^ = code * scale (INT8), code * scale + zero (INT4) never exist as an fp16 tensor, they are
// folded into the dot products in fp32 (FP16-tier rows are used as stored).  A redundant frame's
// entry is a pointer (Algorithm 1), so its source frame's tokens count once more; pruned tokens are
// not in the cache.
//
// One query per head makes Q K^T and P V matrix-vector products: 2 flops per byte read, so the
// kernel is bound by HBM and written as a stream, not for MFMA; the arithmetic is arranged so that
// the vector ALU stays below the memory time (about 5 operations per INT8 element pair instead of
// 12 when every value is first rounded to fp16: the group scale is applied once per row to the dot
// product and to the softmax weight, the INT4 zero-point through sum(q) and a separate accumulator).
// The compressed rows are read once, in pool order (attention does not care about token order),
// with the lane mapping of the pack / unpack kernels: a row is handled by 16 adjacent lanes holding
// 8 consecutive head-dim values each, a 32-value quantisation group is one lane quad, the dot
// product is reduced over the 16 lanes with four DPP moves.  Every lane group keeps an
// online-softmax state (running max, sum and 8 output values per lane); a block merges its 16 lane
// groups through LDS and writes one partial (max, sum, 128 values); a second small kernel merges
// the partials of a head.  The three tiers of a frame are walked by three instances of one loop
// specialised on the row format.

#include "sali_internal.h"

namespace sali {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kRowsPerStep = 4;               // rows in flight per lane group (K and V each)
constexpr int kResidentBlocks = 256 * 8;      // compute units x blocks of the main kernel that fit on one
constexpr int kPartialStride = kAttnPartialStride;   // max, sum, 128 values, padded to whole 128-byte lines

union Row16B {
    u32x4 u;
    _Float16 h[8];
    half2_t h2[4];
};

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

// the lane's piece of the query: 8 values as fp32 and as packed halves, and their sum
struct QueryPiece {
    float f[8];
    half2_t h2[4];
    float sum;
};

// raw piece of one pool row for one lane (16 / 8 / 4 bytes by tier) plus its group's scale and zero
template <int kTier>
struct RawRow;
template <>
struct RawRow<SALI_TIER_FP16> {
    u32x4 u;
};
template <>
struct RawRow<SALI_TIER_INT8> {
    u32x2 u;
    float scale;
};
template <>
struct RawRow<SALI_TIER_INT4> {
    uint32_t u;
    float scale, zero;
};

// prow = row index inside the plane's pool of that tier
__device__ __forceinline__ void load_row(const Pools& pools, size_t plane, size_t prow, int l, RawRow<SALI_TIER_FP16>& r) {
    r.u = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pools.p16) + ((plane * pools.cap16 + prow) * 16 + l));
}
__device__ __forceinline__ void load_row(const Pools& pools, size_t plane, size_t prow, int l, RawRow<SALI_TIER_INT8>& r) {
    const size_t p = plane * pools.cap8 + prow;
    r.u = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(pools.c8 + p * kHeadDim) + l);
    r.scale = pools.s8[p * kGroupsPerRow + (l >> 2)];
}
__device__ __forceinline__ void load_row(const Pools& pools, size_t plane, size_t prow, int l, RawRow<SALI_TIER_INT4>& r) {
    const size_t p = plane * pools.cap4 + prow;
    r.u = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(pools.c4 + p * (kHeadDim / 2)) + l);
    r.scale = pools.s4[p * kGroupsPerRow + (l >> 2)];
    r.zero = (float)__builtin_bit_cast(_Float16, pools.z4[p * kGroupsPerRow + (l >> 2)]);
}

// the lane's part of <q, K^_row>
__device__ __forceinline__ float dot_piece(const RawRow<SALI_TIER_FP16>& r, const QueryPiece& q) {
    Row16B v;
    v.u = r.u;
    float d = 0.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e) d = __builtin_amdgcn_fdot2(q.h2[e], v.h2[e], d, false);
    return d;
}
__device__ __forceinline__ float dot_piece(const RawRow<SALI_TIER_INT8>& r, const QueryPiece& q) {
    float d = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t word = e < 4 ? r.u.x : r.u.y;
        d += q.f[e] * (float)(int)(int8_t)((word >> (8 * (e & 3))) & 0xFF);
    }
    return d * r.scale;
}
__device__ __forceinline__ float dot_piece(const RawRow<SALI_TIER_INT4>& r, const QueryPiece& q) {
    float d = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) d += q.f[e] * (float)((r.u >> (4 * e)) & 0xF);
    return d * r.scale + q.sum * r.zero;
}

// online-softmax state of a lane group (max and sum are equal in its 16 lanes); the INT4
// zero-points are summed apart (zacc, the same for the lane's 8 values) and folded in at the end
struct SoftmaxState {
    float mx, lsum, zacc;
    float acc[8];
};

// acc += p * V^_row for the lane's 8 values
__device__ __forceinline__ void add_value(const RawRow<SALI_TIER_FP16>& r, float p, SoftmaxState& st) {
    Row16B v;
    v.u = r.u;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] += p * (float)v.h[e];
}
__device__ __forceinline__ void add_value(const RawRow<SALI_TIER_INT8>& r, float p, SoftmaxState& st) {
    const float ps = p * r.scale;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t word = e < 4 ? r.u.x : r.u.y;
        st.acc[e] += ps * (float)(int)(int8_t)((word >> (8 * (e & 3))) & 0xFF);
    }
}
__device__ __forceinline__ void add_value(const RawRow<SALI_TIER_INT4>& r, float p, SoftmaxState& st) {
    const float ps = p * r.scale;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] += ps * (float)((r.u >> (4 * e)) & 0xF);
    st.zacc += p * r.zero;
}

// The rows of one tier of one stored frame that fall to this block: 64-row groups split, split +
// n_splits, ...; lane group g takes rows jb + g, jb + 16 + g, ...  `base` = first pool row of the
// frame in this tier, `count` = its rows.
template <int kTier>
__device__ __forceinline__ void attend_tier(const Pools& pools, size_t plane_k, size_t plane_v, int base, int count,
                                            int split, int n_splits, int g, int l, const QueryPiece& q,
                                            float softmax_scale, float mult, SoftmaxState& st) {
    for (int jb = split * 64; jb < count; jb += n_splits * 64) {
        RawRow<kTier> rk[kRowsPerStep], rv[kRowsPerStep];
        bool valid[kRowsPerStep];
#pragma unroll
        for (int r = 0; r < kRowsPerStep; ++r) {
            const int j = jb + r * 16 + g;
            valid[r] = j < count;
            rk[r] = {};
            rv[r] = {};
            if (valid[r]) {
                load_row(pools, plane_k, (size_t)(base + j), l, rk[r]);
                load_row(pools, plane_v, (size_t)(base + j), l, rv[r]);
            }
        }
        float s[kRowsPerStep];
        float bm = -INFINITY;
#pragma unroll
        for (int r = 0; r < kRowsPerStep; ++r) {
            const float d = row16_sum(dot_piece(rk[r], q));
            s[r] = valid[r] ? softmax_scale * d : -INFINITY;
            bm = fmaxf(bm, s[r]);
        }
        const float new_mx = fmaxf(st.mx, bm);
        if (new_mx == -INFINITY) continue;          // no row for this lane group yet (uniform inside it)
        const float corr = __expf(st.mx - new_mx);  // first rows: exp(-inf) = 0
        st.lsum *= corr;
        st.zacc *= corr;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[e] *= corr;
#pragma unroll
        for (int r = 0; r < kRowsPerStep; ++r) {
            const float p = mult * __expf(s[r] - new_mx);   // absent row: exp(-inf) = 0
            st.lsum += p;
            add_value(rv[r], p, st);
        }
        st.mx = new_mx;
    }
}

}  // namespace

// grid (n_chunks * n_splits, n_heads).  Block (c, s) of head h takes the frames
// [frame_lo + c * frames_per_chunk, ...) and of each source frame the 64-row groups s, s + n_splits, ...
// of every tier, and writes one partial.
__global__ __launch_bounds__(256) void k_attn_partial(const sali_frame_row* __restrict__ rows, Pools pools, int layer,
                                                      int n_heads, const _Float16* __restrict__ q, int frame_lo,
                                                      int frame_hi, int frames_per_chunk, int n_splits,
                                                      float softmax_scale, float* __restrict__ partial) {
    __shared__ float s_m[16], s_l[16];
    __shared__ float s_acc[16][kHeadDim];

    const int h = blockIdx.y;
    const int chunk = blockIdx.x / n_splits, split = blockIdx.x % n_splits;
    const int g = threadIdx.x >> 4, l = threadIdx.x & 15;
    const size_t plane_k = ((size_t)layer * 2 + 0) * n_heads + h;
    const size_t plane_v = ((size_t)layer * 2 + 1) * n_heads + h;

    QueryPiece qp;
    {
        Row16B qv;
        qv.u = reinterpret_cast<const u32x4*>(q)[h * 16 + l];
        qp.sum = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            qp.f[e] = (float)qv.h[e];
            qp.sum += qp.f[e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) qp.h2[e] = qv.h2[e];
    }

    SoftmaxState st;
    st.mx = -INFINITY;
    st.lsum = 0.0f;
    st.zacc = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] = 0.0f;

    const int f0 = frame_lo + chunk * frames_per_chunk;
    const int f1 = min(frame_hi, f0 + frames_per_chunk);
    for (int f = f0; f < f1; ++f) {
        // Which stored frame does frame f bring in, and how many times?  A stored frame counts for
        // itself and for the redundant frames behind it (up to the next stored frame or the end of
        // the range); redundant frames at the head of the range, whose source lies before it, are
        // counted at the first of them.  Every thread takes the same decision from the same
        // (uniform) table reads.
        const sali_frame_row r = rows[f];
        bool leader = r.stored != 0;
        if (!leader && r.src >= 0 && r.src < frame_lo) {
            leader = true;
            for (int t = frame_lo; t < f; ++t)
                if (rows[t].src == r.src) leader = false;          // an earlier frame of the run counts them
        }
        if (!leader) continue;
        const int src = r.src;
        int n_uses = 1;
        for (int t = f + 1; t < frame_hi && rows[t].stored == 0; ++t)
            if (rows[t].src == src) ++n_uses;
        const float mult = (float)n_uses;
        const sali_frame_row row = rows[src];
        attend_tier<SALI_TIER_FP16>(pools, plane_k, plane_v, row.base16, row.n16, split, n_splits, g, l, qp,
                                    softmax_scale, mult, st);
        attend_tier<SALI_TIER_INT8>(pools, plane_k, plane_v, row.base8, row.n8, split, n_splits, g, l, qp,
                                    softmax_scale, mult, st);
        attend_tier<SALI_TIER_INT4>(pools, plane_k, plane_v, row.base4, row.n4, split, n_splits, g, l, qp,
                                    softmax_scale, mult, st);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] += st.zacc;

    // merge the 16 lane groups
    if (l == 0) {
        s_m[g] = st.mx;
        s_l[g] = st.lsum;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_acc[g][8 * l + e] = st.acc[e];
    __syncthreads();
    float* mine = partial + ((size_t)h * kAttnPartials + blockIdx.x) * kPartialStride;
    if (threadIdx.x < kHeadDim) {
        float big = -INFINITY;
#pragma unroll
        for (int k = 0; k < 16; ++k) big = fmaxf(big, s_m[k]);
        float lt = 0.0f, at = 0.0f;
        if (big != -INFINITY) {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const float w = __expf(s_m[k] - big);
                lt += w * s_l[k];
                at += w * s_acc[k][threadIdx.x];
            }
        }
        if (threadIdx.x == 0) {
            mine[0] = big;
            mine[1] = lt;
        }
        mine[2 + threadIdx.x] = at;
    }
}

// grid (n_heads), 256 threads: merge of a head's partials (n_partials <= kAttnPartials; 0 for an
// empty frame range: zeros and -inf).  A kernel of its own: the kernel boundary is the only
// device-wide ordering this needs, and a device-scope fence in each of the ~2000 blocks of the
// main kernel (last-block hand-over) measured 4.5x slower, because on this chip such a fence writes
// back and invalidates the L2 of the issuing XCD under the stream that the other blocks are reading.
__global__ __launch_bounds__(256) void k_attn_merge(const float* __restrict__ partial, int n_partials,
                                                    float* __restrict__ out, float* __restrict__ lse) {
    __shared__ float s_w[kAttnPartials];
    __shared__ float s_part[2][kHeadDim];
    const int h = blockIdx.x;
    const float* p = partial + (size_t)h * kAttnPartials * kPartialStride;
    for (int k = threadIdx.x; k < n_partials; k += 256) s_w[k] = p[(size_t)k * kPartialStride];
    __syncthreads();
    float big = -INFINITY;
    for (int k = 0; k < n_partials; ++k) big = fmaxf(big, s_w[k]);
    __syncthreads();
    for (int k = threadIdx.x; k < n_partials; k += 256) s_w[k] = big != -INFINITY ? expf(s_w[k] - big) : 0.0f;
    __syncthreads();
    // the two halves of the block take alternate partials; thread d of a half sums output value d
    const int d = threadIdx.x & (kHeadDim - 1), half = threadIdx.x >> 7;
    float lt = 0.0f, at = 0.0f;
#pragma unroll 8
    for (int k = half; k < n_partials; k += 2) {
        const float w = s_w[k];
        lt += w * p[(size_t)k * kPartialStride + 1];
        at += w * p[(size_t)k * kPartialStride + 2 + d];
    }
    if (half == 1) {
        s_part[0][d] = at;
        s_part[1][d] = lt;
    }
    __syncthreads();
    if (half == 0) {
        at += s_part[0][d];
        lt += s_part[1][d];
        out[h * kHeadDim + d] = lt > 0.0f ? at / lt : 0.0f;
        if (lse != nullptr && d == 0) lse[h] = lt > 0.0f ? big + logf(lt) : -INFINITY;
    }
}

hipError_t launch_attend(const sali_frame_row* d_rows, Pools pools, int layer, int n_heads, const void* d_q,
                         int frame_lo, int frame_hi, float softmax_scale, float* d_partial, float* d_out,
                         float* d_lse_or_null, hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t s) {
    const int n_range = frame_hi - frame_lo;
    int n_partials = 0;
    if (n_range > 0) {
        // One resident round of blocks: at 8 blocks of 256 threads per compute unit the chip holds
        // kResidentBlocks; more blocks than that leave a second, nearly empty round at the end of a
        // bandwidth-bound kernel.  Blocks of a head: whole frames per block for long ranges, row
        // groups of a frame split over blocks for short ones (up to 9 groups of 64 rows per tier).
        int per_head = kResidentBlocks / n_heads;
        per_head = per_head < 1 ? 1 : (per_head > kAttnPartials ? kAttnPartials : per_head);
        const int fpc = (n_range + per_head - 1) / per_head;
        const int n_chunks = (n_range + fpc - 1) / fpc;
        int n_splits = per_head / n_chunks;
        n_splits = n_splits < 1 ? 1 : (n_splits > 9 ? 9 : n_splits);
        n_partials = n_chunks * n_splits;
        if (ev_start != nullptr && hipEventRecord(ev_start, s) != hipSuccess) return hipErrorUnknown;
        hipLaunchKernelGGL(k_attn_partial, dim3(n_partials, n_heads), dim3(256), 0, s, d_rows, pools, layer, n_heads,
                           reinterpret_cast<const _Float16*>(d_q), frame_lo, frame_hi, fpc, n_splits, softmax_scale,
                           d_partial);
        if (ev_stop != nullptr && hipEventRecord(ev_stop, s) != hipSuccess) return hipErrorUnknown;
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_attn_merge, dim3(n_heads), dim3(256), 0, s, d_partial, n_partials, d_out, d_lse_or_null);
    return hipGetLastError();
}

}  // namespace sali
