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
// specialised on the row format.  With grouped-query attention the kQ query heads that share a K/V
// head are handled by the same block, so every compressed row is still read once.

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

// frow = row index in the flat pool array of that tier (pool_row0 of the frame and plane + the row
// inside the frame's run)
__device__ __forceinline__ void load_row(const Pools& pools, size_t frow, int l, RawRow<SALI_TIER_FP16>& r) {
    r.u = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pools.p16) + (frow * 16 + l));
}
__device__ __forceinline__ void load_row(const Pools& pools, size_t frow, int l, RawRow<SALI_TIER_INT8>& r) {
    r.u = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(pools.c8 + frow * kHeadDim) + l);
    r.scale = pools.s8[frow * kGroupsPerRow + (l >> 2)];
}
__device__ __forceinline__ void load_row(const Pools& pools, size_t frow, int l, RawRow<SALI_TIER_INT4>& r) {
    r.u = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(pools.c4 + frow * (kHeadDim / 2)) + l);
    r.scale = pools.s4[frow * kGroupsPerRow + (l >> 2)];
    r.zero = (float)__builtin_bit_cast(_Float16, pools.z4[frow * kGroupsPerRow + (l >> 2)]);
}

// The lane's 8 stored values of a row as fp32: the halves of an FP16 row, the raw codes of an
// INT8 / INT4 row (scale and zero-point are applied once per row, see finish_dot / weight_of).
__device__ __forceinline__ void row_values(const RawRow<SALI_TIER_FP16>& r, float x[8]) {
    Row16B v;
    v.u = r.u;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (float)v.h[e];
}
__device__ __forceinline__ void row_values(const RawRow<SALI_TIER_INT8>& r, float x[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t word = e < 4 ? r.u.x : r.u.y;
        x[e] = (float)(int)(int8_t)((word >> (8 * (e & 3))) & 0xFF);
    }
}
__device__ __forceinline__ void row_values(const RawRow<SALI_TIER_INT4>& r, float x[8]) {
    // nibbles to bytes first (even elements in one word, odd ones in the other): a byte converts to fp32
    // in one instruction; the empty asm keeps the compiler from folding the bytes back into nibbles
    uint32_t ev = r.u & 0x0F0F0F0Fu, od = (r.u >> 4) & 0x0F0F0F0Fu;
    asm volatile("" : "+v"(ev), "+v"(od));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = (float)((ev >> (8 * i)) & 0xFFu);
        x[2 * i + 1] = (float)((od >> (8 * i)) & 0xFFu);
    }
}

// <q, K^_row> of the lane from the sum over its raw values: K^ = code * scale (+ zero)
__device__ __forceinline__ float finish_dot(const RawRow<SALI_TIER_FP16>&, float d, const QueryPiece&) { return d; }
__device__ __forceinline__ float finish_dot(const RawRow<SALI_TIER_INT8>& r, float d, const QueryPiece&) {
    return d * r.scale;
}
__device__ __forceinline__ float finish_dot(const RawRow<SALI_TIER_INT4>& r, float d, const QueryPiece& q) {
    return d * r.scale + q.sum * r.zero;
}

// p * V^_row = (p * scale) * code + p * zero: weight on the raw values, and the constant part
__device__ __forceinline__ float weight_of(const RawRow<SALI_TIER_FP16>&, float p) { return p; }
__device__ __forceinline__ float weight_of(const RawRow<SALI_TIER_INT8>& r, float p) { return p * r.scale; }
__device__ __forceinline__ float weight_of(const RawRow<SALI_TIER_INT4>& r, float p) { return p * r.scale; }
__device__ __forceinline__ float offset_of(const RawRow<SALI_TIER_FP16>&, float) { return 0.0f; }
__device__ __forceinline__ float offset_of(const RawRow<SALI_TIER_INT8>&, float) { return 0.0f; }
__device__ __forceinline__ float offset_of(const RawRow<SALI_TIER_INT4>& r, float p) { return p * r.zero; }

// online-softmax state of a lane group for one query (max and sum are equal in its 16 lanes); the
// INT4 zero-points are summed apart (zacc, the same for the lane's 8 values) and folded in at the end
struct SoftmaxState {
    float mx, lsum, zacc;
    float acc[8];
};

// The rows of one tier of one stored frame that fall to this block: 64-row groups split, split +
// n_splits, ...; lane group g takes rows jb + g, jb + 16 + g, ...  `base` = first pool row of the
// frame in this tier, `count` = its rows.  kQ queries share every row that is read.
template <int kTier, int kQ>
__device__ __forceinline__ void attend_tier(const Pools& pools, size_t plane_k, size_t plane_v, int base, int count,
                                            int split, int n_splits, int g, int l, const QueryPiece (&q)[kQ],
                                            float softmax_scale, float mult, SoftmaxState (&st)[kQ]) {
    const size_t row0_k = pool_row0(pools, base, count, plane_k), row0_v = pool_row0(pools, base, count, plane_v);
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
                load_row(pools, row0_k + (size_t)j, l, rk[r]);
                load_row(pools, row0_v + (size_t)j, l, rv[r]);
            }
        }
        float s[kQ][kRowsPerStep];
#pragma unroll
        for (int r = 0; r < kRowsPerStep; ++r) {
            float x[8];
            row_values(rk[r], x);
#pragma unroll
            for (int iq = 0; iq < kQ; ++iq) {
                float d = 0.0f;
                if constexpr (kTier == SALI_TIER_FP16) {
                    Row16B v;
                    v.u = rk[r].u;
#pragma unroll
                    for (int e = 0; e < 4; ++e) d = __builtin_amdgcn_fdot2(q[iq].h2[e], v.h2[e], d, false);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) d += q[iq].f[e] * x[e];
                }
                d = row16_sum(finish_dot(rk[r], d, q[iq]));
                s[iq][r] = valid[r] ? softmax_scale * d : -INFINITY;
            }
        }
        float p[kQ][kRowsPerStep];
#pragma unroll
        for (int iq = 0; iq < kQ; ++iq) {
            float bm = -INFINITY;
#pragma unroll
            for (int r = 0; r < kRowsPerStep; ++r) bm = fmaxf(bm, s[iq][r]);
            const float new_mx = fmaxf(st[iq].mx, bm);
            // nothing seen yet for this lane group: keep the state (every weight below is exp(-inf) = 0,
            // and the reference maximum must stay finite for that)
            const float ref = new_mx == -INFINITY ? 0.0f : new_mx;
            const float corr = __expf(st[iq].mx - ref);     // first rows: exp(-inf) = 0
            st[iq].lsum *= corr;
            st[iq].zacc *= corr;
#pragma unroll
            for (int e = 0; e < 8; ++e) st[iq].acc[e] *= corr;
#pragma unroll
            for (int r = 0; r < kRowsPerStep; ++r) {
                p[iq][r] = mult * __expf(s[iq][r] - ref);   // absent row: exp(-inf) = 0
                st[iq].lsum += p[iq][r];
            }
            st[iq].mx = new_mx;
        }
#pragma unroll
        for (int r = 0; r < kRowsPerStep; ++r) {
            float x[8];
            row_values(rv[r], x);
#pragma unroll
            for (int iq = 0; iq < kQ; ++iq) {
                const float wgt = weight_of(rv[r], p[iq][r]);
                st[iq].zacc += offset_of(rv[r], p[iq][r]);
#pragma unroll
                for (int e = 0; e < 8; ++e) st[iq].acc[e] += wgt * x[e];
            }
        }
    }
}

}  // namespace

// grid (n_chunks * n_splits, n_heads).  Block (c, s) of K/V head h takes the frames
// [frame_lo + c * frames_per_chunk, ...) and of each source frame the 64-row groups s, s + n_splits, ...
// of every tier, for kQ of the query heads that share the K/V head (gridDim.z such sets:
// q_per_kv = kQ * gridDim.z), and writes one partial per query head.
template <int kQ>
__global__ __launch_bounds__(256) void k_attn_partial(const sali_frame_row* __restrict__ rows, Pools pools, int layer,
                                                      int n_heads, const _Float16* __restrict__ q, int frame_lo,
                                                      int frame_hi, int frames_per_chunk, int n_splits,
                                                      float softmax_scale, float* __restrict__ partial) {
    __shared__ float s_m[16], s_l[16];
    __shared__ float s_acc[16][kHeadDim];

    const int h = blockIdx.y;
    const int q_first = (h * (int)gridDim.z + (int)blockIdx.z) * kQ;      // first query head of this block
    const int chunk = blockIdx.x / n_splits, split = blockIdx.x % n_splits;
    const int g = threadIdx.x >> 4, l = threadIdx.x & 15;
    const size_t plane_k = ((size_t)layer * 2 + 0) * n_heads + h;
    const size_t plane_v = ((size_t)layer * 2 + 1) * n_heads + h;

    QueryPiece qp[kQ];
    SoftmaxState st[kQ];
#pragma unroll
    for (int iq = 0; iq < kQ; ++iq) {
        Row16B qv;
        qv.u = reinterpret_cast<const u32x4*>(q)[(q_first + iq) * 16 + l];
        qp[iq].sum = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            qp[iq].f[e] = (float)qv.h[e];
            qp[iq].sum += qp[iq].f[e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) qp[iq].h2[e] = qv.h2[e];
        st[iq].mx = -INFINITY;
        st[iq].lsum = 0.0f;
        st[iq].zacc = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st[iq].acc[e] = 0.0f;
    }

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
        attend_tier<SALI_TIER_FP16, kQ>(pools, plane_k, plane_v, row.base16, row.n16, split, n_splits, g, l, qp,
                                        softmax_scale, mult, st);
        attend_tier<SALI_TIER_INT8, kQ>(pools, plane_k, plane_v, row.base8, row.n8, split, n_splits, g, l, qp,
                                        softmax_scale, mult, st);
        attend_tier<SALI_TIER_INT4, kQ>(pools, plane_k, plane_v, row.base4, row.n4, split, n_splits, g, l, qp,
                                        softmax_scale, mult, st);
    }

    // merge the 16 lane groups, one query head after the other
#pragma unroll
    for (int iq = 0; iq < kQ; ++iq) {
        if (iq > 0) __syncthreads();
        if (l == 0) {
            s_m[g] = st[iq].mx;
            s_l[g] = st[iq].lsum;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) s_acc[g][8 * l + e] = st[iq].acc[e] + st[iq].zacc;
        __syncthreads();
        float* mine = partial + ((size_t)(q_first + iq) * kAttnPartials + blockIdx.x) * kPartialStride;
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
}

// grid (n_heads), 256 threads: merge of a head's partials (n_partials <= kAttnPartials; 0 for an
// empty frame range: zeros and -inf).  A kernel of its own: the kernel boundary is the only
// device-wide ordering this needs, and a device-scope fence in each of the ~2000 blocks of the
// main kernel (last-block hand-over) measured 4.5x slower, because on this chip such a fence writes
// back and invalidates the L2 of the issuing XCD under the stream that the other blocks are reading.
__global__ __launch_bounds__(256) void k_attn_merge(const float* __restrict__ partial, int n_partials, int slots,
                                                    float* __restrict__ out, float* __restrict__ lse) {
    __shared__ float s_w[kAttnPartials];
    __shared__ float s_part[2][kHeadDim];
    const int h = blockIdx.x;
    const float* p = partial + (size_t)h * slots * kPartialStride;      // `slots` partials are reserved per query head
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

// ---------------------------------------------------------------------------------------------
// Many queries per K/V head (16, 32 or 64: the tokens of a prompt attending to the cached video, or
// large query groups): Q K^T and P V are real matrix products, so they run on the matrix cores
// (v_mfma_f32_32x32x16_f16) and every compressed row is still read once for all queries.
//
// One wave = one work item (a chunk of frames x a row split, as in the single-query kernel) x one
// K/V head x one tile of 32 queries; the four waves of a block share the 32 queries (LDS).  Per tile
// of 32 cached rows:
//   S^T = K^ Q^T : A operand = K^ tile (lane = row n, registers = head-dim values), B operand = the
//        queries (lane = query m); the result has lane = query, registers = rows, so the softmax
//        over rows is a reduction over the lane's 16 registers and one exchange between the two
//        lane halves, and P in that layout IS the B operand of the second product (the rows of the
//        tile are contracted in the order the registers hold them);
//   out^T = V^^T P^T : A operand = V^^T (lane = head-dim value d, registers = two runs of 4
//        consecutive rows), read column-wise from the wave's LDS tile, which holds K^ first and V^ after.
// The head-dim index of the contraction is permuted (lane half hh of a row holds values
// [64 hh, 64 hh + 64), k-step t takes 8 of them from each half) so that a lane reads one contiguous
// piece of its row; Q uses the same permutation.  Here the dequantised values DO exist as fp16
// (K^ = fp16(code * scale), fp16(code * scale + zero), the values dequantise-on-read produces) because
// the matrix cores take fp16 operands; the softmax weights are rounded to fp16 for the second product
// as well.  Both stay inside the tolerance of the floating-point results (largest error printed by
// the tests).  Accumulation, softmax state and partials are fp32; partials have the layout of the
// single-query kernel and are merged by the same k_attn_merge.
// The kernel is bound by instruction issue (conversions of the codes, softmax, LDS traffic and the
// matrix instructions of a tile share one SIMD): one, two or three resident waves per SIMD take the
// same time, and so do 16 and 32 queries.
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

namespace {

constexpr int kPfRows = 32;                       // cached rows per tile
constexpr int kPfVStride = kHeadDim + 8;          // halves per LDS row of a tile (skewed against bank conflicts)
constexpr int kPfWavesPerSimd = 2;                // resident waves the launch is sized for

union Half8 {
    u32x4 u;
    half4_t h4[2];
    _Float16 h[8];
};

// A tile of 32 pool rows is read with fully coalesced 16-byte loads (consecutive lanes read
// consecutive memory: a lane-per-row pattern, which the matrix-core operands would suggest, was
// measured at 1.6 TB/s), dequantised to fp16 where it lies, and written to the wave's LDS tile
// [32 rows][128 values]; the operands are then read from LDS in the layout the instruction wants.
// Piece `idx` of a tile = 16 bytes of row idx / (pieces per row).  Rows past the end of the run
// repeat its last row (their softmax weight is zero).
template <int kTier>
struct PfRaw;
template <>
struct PfRaw<SALI_TIER_FP16> {
    u32x4 c[8];                 // 8 values each
};
template <>
struct PfRaw<SALI_TIER_INT8> {
    u32x4 c[4];                 // 16 codes each
    float sc[4];
};
template <>
struct PfRaw<SALI_TIER_INT4> {
    u32x4 c[2];                 // 32 codes each = one quantisation group
    float sc[2], zp[2];
};

__device__ __forceinline__ void pf_load_tile(const Pools& pools, size_t row0, int jb, int count, int lane,
                                             PfRaw<SALI_TIER_FP16>& r) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int idx = u * 64 + lane;
        const size_t frow = row0 + (size_t)min(jb + (idx >> 4), count - 1);
        r.c[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pools.p16 + frow * kHeadDim) + (idx & 15));
    }
}
__device__ __forceinline__ void pf_load_tile(const Pools& pools, size_t row0, int jb, int count, int lane,
                                             PfRaw<SALI_TIER_INT8>& r) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int idx = u * 64 + lane;
        const size_t frow = row0 + (size_t)min(jb + (idx >> 3), count - 1);
        r.c[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pools.c8 + frow * kHeadDim) + (idx & 7));
        r.sc[u] = pools.s8[frow * kGroupsPerRow + ((idx & 7) >> 1)];
    }
}
__device__ __forceinline__ void pf_load_tile(const Pools& pools, size_t row0, int jb, int count, int lane,
                                             PfRaw<SALI_TIER_INT4>& r) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int idx = u * 64 + lane;
        const size_t frow = row0 + (size_t)min(jb + (idx >> 2), count - 1);
        r.c[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pools.c4 + frow * (kHeadDim / 2)) + (idx & 3));
        r.sc[u] = pools.s4[frow * kGroupsPerRow + (idx & 3)];
        r.zp[u] = (float)__builtin_bit_cast(_Float16, pools.z4[frow * kGroupsPerRow + (idx & 3)]);
    }
}

// dequantise the lane's pieces and put them where they belong in the LDS tile
__device__ __forceinline__ void pf_store_tile(const PfRaw<SALI_TIER_FP16>& r, int lane, _Float16 (*tile)[kPfVStride]) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int idx = u * 64 + lane;
        *reinterpret_cast<u32x4*>(&tile[idx >> 4][8 * (idx & 15)]) = r.c[u];
    }
}
__device__ __forceinline__ void pf_store_tile(const PfRaw<SALI_TIER_INT8>& r, int lane, _Float16 (*tile)[kPfVStride]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int idx = u * 64 + lane;
        Half8 o[2];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const uint32_t word = w == 0 ? r.c[u].x : (w == 1 ? r.c[u].y : (w == 2 ? r.c[u].z : r.c[u].w));
#pragma unroll
            for (int i = 0; i < 4; ++i)
                o[w >> 1].h[4 * (w & 1) + i] = (_Float16)((float)(int)(int8_t)((word >> (8 * i)) & 0xFF) * r.sc[u]);
        }
        u32x4* dst = reinterpret_cast<u32x4*>(&tile[idx >> 3][16 * (idx & 7)]);
        dst[0] = o[0].u;
        dst[1] = o[1].u;
    }
}
__device__ __forceinline__ void pf_store_tile(const PfRaw<SALI_TIER_INT4>& r, int lane, _Float16 (*tile)[kPfVStride]) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int idx = u * 64 + lane;
        u32x4* dst = reinterpret_cast<u32x4*>(&tile[idx >> 2][32 * (idx & 3)]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {                               // 8 values = one word of codes
            const uint32_t word = w == 0 ? r.c[u].x : (w == 1 ? r.c[u].y : (w == 2 ? r.c[u].z : r.c[u].w));
            // nibbles to bytes first (even elements in one word, odd ones in another): a byte converts to
            // fp32 in one instruction, a nibble needs a shift and a mask each
            uint32_t ev = word & 0x0F0F0F0Fu, od = (word >> 4) & 0x0F0F0F0Fu;
            asm volatile("" : "+v"(ev), "+v"(od));      // (keeps the compiler from folding the bytes back into nibbles)
            Half8 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                o.h[2 * i] = (_Float16)__builtin_fmaf((float)((ev >> (8 * i)) & 0xFFu), r.sc[u], r.zp[u]);
                o.h[2 * i + 1] = (_Float16)__builtin_fmaf((float)((od >> (8 * i)) & 0xFFu), r.sc[u], r.zp[u]);
            }
            dst[w] = o.u;
        }
    }
}

struct PfState {
    float mx, lsum;
    float16_t acc[4];           // acc[dt][r] = out[m][32 dt + 8 (r / 4) + 4 hh + r % 4], not yet normalised
};

// LDS operations of one wave execute in order, so the wave's private tiles need no barrier, only
// that the compiler keeps the order
__device__ __forceinline__ void pf_lds_order() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// the tiles of one tier of one stored frame that fall to this wave
template <int kTier>
__device__ __forceinline__ void pf_tier(const Pools& pools, size_t plane_k, size_t plane_v, int base, int count,
                                        int split, int n_splits, int lane, const _Float16 (*s_q)[kPfVStride],
                                        float softmax_scale, float mult, _Float16 (*s_t)[kPfVStride], PfState& st) {
    const int m = lane & 31, hh = lane >> 5;
    const size_t row0_k = pool_row0(pools, base, count, plane_k), row0_v = pool_row0(pools, base, count, plane_v);
    // Software pipeline: the loads of the next tile are in flight while this one is worked on (K^ rows
    // are asked for as soon as this tile's K^ registers have gone to LDS, V^ rows likewise), and they are
    // issued without a branch: past the end of the run every row index clamps to the run's last row, one
    // cache line.  Without it the waves of the chip run in step, all waiting for memory and then all
    // computing, and the kernel takes the sum of the two times instead of the larger.
    const int step = n_splits * kPfRows;
    int jb = split * kPfRows;
    if (jb >= count) return;
    PfRaw<kTier> rk, rv;
    pf_load_tile(pools, row0_k, jb, count, lane, rk);
    pf_load_tile(pools, row0_v, jb, count, lane, rv);
    for (; jb < count; jb += step) {
        pf_lds_order();                                            // the previous tile's reads are done
        pf_store_tile(rk, lane, s_t);
        pf_lds_order();
        pf_load_tile(pools, row0_k, jb + step, count, lane, rk);
        // S^T = K^ Q^T with v_mfma_f32_32x32x16_f16 (A[i][k]: lane = i + 32 (k / 8), element k % 8; B alike;
        // D[i][j]: lane = j + 32 hh, register r holds i = 8 (r / 4) + 4 hh + r % 4).  Lane (row m, half hh),
        // step t: values 64 hh + 8 t .. + 7 of the row; the queries use the same assignment
        float16_t s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.0f;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const half8_t ka = *reinterpret_cast<const half8_t*>(&s_t[m][64 * hh + 8 * t]);
            const half8_t qb = *reinterpret_cast<const half8_t*>(&s_q[m][64 * hh + 8 * t]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_f16(ka, qb, s, 0, 0, 0);
        }
        // s[r] = <K^ row jb + n(r), query m>, n(r) = 8 (r / 4) + 4 hh + r % 4
        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int n = 8 * (r / 4) + 4 * hh + (r % 4);
            s[r] = (jb + n < count) ? s[r] * softmax_scale : -INFINITY;
            tmax = fmaxf(tmax, s[r]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float mnew = fmaxf(st.mx, tmax);
        const float corr = __expf(st.mx - mnew);
        float psum = 0.0f;
        // the softmax weights in the order the second product wants them: step jj of two, element e of the
        // lane's eight = row 16 jj + 8 (e / 4) + 4 hh + e % 4 of the tile, which is register 8 jj + e
        half8_t pb[2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float p = mult * __expf(s[8 * jj + e] - mnew);
                psum += p;
                pb[jj][e] = (_Float16)p;
            }
        psum += __shfl_xor(psum, 32);
        st.lsum = st.lsum * corr + psum;
        st.mx = mnew;
        // the 64 accumulators are rescaled only when some query of the wave saw a new maximum (rare after
        // the first tiles); the test is wave-uniform
        if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.acc[dt][r] *= corr;
        }
        // out^T += V^^T P^T: A operand lane (value d = 32 dt + m, half hh): the same eight rows of column d
        pf_lds_order();                                            // the K^ reads come first: same tile
        pf_store_tile(rv, lane, s_t);
        pf_lds_order();
        pf_load_tile(pools, row0_v, jb + step, count, lane, rv);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                half8_t va;
#pragma unroll
                for (int e = 0; e < 8; ++e) va[e] = s_t[16 * jj + 8 * (e / 4) + 4 * hh + (e % 4)][32 * dt + m];
                st.acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va, pb[jj], st.acc[dt], 0, 0, 0);
            }
    }
}

}  // namespace

// grid (ceil(n_partials / 4), n_heads, ceil(q_per_kv / 32)), 256 threads = four independent waves
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_prefill(const sali_frame_row* __restrict__ rows, Pools pools, int layer,
                                                      int n_heads, const _Float16* __restrict__ q, int q_per_kv,
                                                      int frame_lo, int frame_hi, int frames_per_chunk, int n_splits,
                                                      int n_partials, float softmax_scale, float* __restrict__ partial) {
    __shared__ __align__(16) _Float16 s_q[32][kPfVStride];               // the block's 32 queries (zeros past q_per_kv)
    __shared__ __align__(16) _Float16 s_t_all[4][kPfRows][kPfVStride];   // one K^ / V^ tile per wave
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = lane & 31, hh = lane >> 5;
    const int h = blockIdx.y;
    for (int idx = threadIdx.x; idx < 32 * 16; idx += 256) {
        const int qrow = idx >> 4, piece = idx & 15;
        const int qq = (int)blockIdx.z * 32 + qrow;
        u32x4 v = (u32x4){0u, 0u, 0u, 0u};
        if (qq < q_per_kv) v = reinterpret_cast<const u32x4*>(q + ((size_t)h * q_per_kv + qq) * kHeadDim)[piece];
        *reinterpret_cast<u32x4*>(&s_q[qrow][8 * piece]) = v;
    }
    __syncthreads();
    const int item = (int)blockIdx.x * 4 + wave;
    if (item >= n_partials) return;
    const int chunk = item / n_splits, split = item % n_splits;
    const int qi = (int)blockIdx.z * 32 + m;                 // this lane's query among the q_per_kv of the K/V head
    const bool q_valid = qi < q_per_kv;
    const size_t q_head = (size_t)h * q_per_kv + (q_valid ? qi : 0);
    const size_t plane_k = ((size_t)layer * 2 + 0) * n_heads + h;
    const size_t plane_v = ((size_t)layer * 2 + 1) * n_heads + h;

    PfState st;
    st.mx = -INFINITY;
    st.lsum = 0.0f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.acc[dt][r] = 0.0f;

    const int f0 = frame_lo + chunk * frames_per_chunk;
    const int f1 = min(frame_hi, f0 + frames_per_chunk);
    for (int f = f0; f < f1; ++f) {
        // which stored frame frame f brings in, and how often: as in k_attn_partial
        const sali_frame_row r = rows[f];
        bool leader = r.stored != 0;
        if (!leader && r.src >= 0 && r.src < frame_lo) {
            leader = true;
            for (int t = frame_lo; t < f; ++t)
                if (rows[t].src == r.src) leader = false;
        }
        if (!leader) continue;
        const int src = r.src;
        int n_uses = 1;
        for (int t = f + 1; t < frame_hi && rows[t].stored == 0; ++t)
            if (rows[t].src == src) ++n_uses;
        const float mult = (float)n_uses;
        const sali_frame_row row = rows[src];
        pf_tier<SALI_TIER_FP16>(pools, plane_k, plane_v, row.base16, row.n16, split, n_splits, lane, s_q, softmax_scale, mult,
                                s_t_all[wave], st);
        pf_tier<SALI_TIER_INT8>(pools, plane_k, plane_v, row.base8, row.n8, split, n_splits, lane, s_q, softmax_scale, mult,
                                s_t_all[wave], st);
        pf_tier<SALI_TIER_INT4>(pools, plane_k, plane_v, row.base4, row.n4, split, n_splits, lane, s_q, softmax_scale, mult,
                                s_t_all[wave], st);
    }
    if (!q_valid) return;
    float* mine = partial + (q_head * (size_t)n_partials + item) * kPartialStride;
    if (hh == 0) {
        mine[0] = st.mx;
        mine[1] = st.lsum;
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[2 + 32 * dt + 8 * (r / 4) + 4 * hh + (r % 4)] = st.acc[dt][r];
}

hipError_t launch_attend(const sali_frame_row* d_rows, Pools pools, int layer, int n_heads, int q_per_kv,
                         const void* d_q, int frame_lo, int frame_hi, float softmax_scale, float* d_partial,
                         float* d_out, float* d_lse_or_null, hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t s) {
    const int n_range = frame_hi - frame_lo;
    int n_partials = 0;
    if (n_range > 0 && q_per_kv > kAttnMaxQPerKv) {
        // matrix-core path: 32 queries per wave; the scratch holds kAttnSlotsPerHead partials per K/V head,
        // shared out over the q_per_kv query heads
        // and one resident round of waves (kPfWavesPerSimd per SIMD: 2048 on the chip) is the target, as for the streaming kernel
        int per_head = kAttnSlotsPerHead / q_per_kv;
        const int round = (kPfWavesPerSimd * 4 * 256) / (n_heads * ((q_per_kv + 31) / 32));
        per_head = per_head > round ? (round < 1 ? 1 : round) : per_head;
        per_head = per_head > kAttnPartials ? kAttnPartials : per_head;
        // work items = chunks of whole frames x row splits inside a frame; of the few ways to get close to
        // per_head items take the one with the most items
        int fpc = (n_range + per_head - 1) / per_head, n_chunks = 0, n_splits = 0;
        for (int cand = fpc; cand <= fpc + 3; ++cand) {
            const int chunks = (n_range + cand - 1) / cand;
            int splits = per_head / chunks;
            splits = splits < 1 ? 1 : (splits > kTokens / kPfRows ? kTokens / kPfRows : splits);
            if (chunks * splits > n_chunks * n_splits && chunks * splits <= per_head) {
                fpc = cand;
                n_chunks = chunks;
                n_splits = splits;
            }
        }
        if (n_chunks == 0) {            // per_head below the number of chunks cannot happen (fpc covers the range)
            n_chunks = (n_range + fpc - 1) / fpc;
            n_splits = 1;
        }
        n_partials = n_chunks * n_splits;
        if (ev_start != nullptr && hipEventRecord(ev_start, s) != hipSuccess) return hipErrorUnknown;
        const dim3 grid((n_partials + 3) / 4, n_heads, (q_per_kv + 31) / 32);
        hipLaunchKernelGGL(k_attn_prefill, grid, dim3(256), 0, s, d_rows, pools, layer, n_heads,
                           reinterpret_cast<const _Float16*>(d_q), q_per_kv, frame_lo, frame_hi, fpc, n_splits, n_partials,
                           softmax_scale, d_partial);
        if (ev_stop != nullptr && hipEventRecord(ev_stop, s) != hipSuccess) return hipErrorUnknown;
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_attn_merge, dim3(n_heads * q_per_kv), dim3(256), 0, s, d_partial, n_partials, n_partials,
                           d_out, d_lse_or_null);
        return hipGetLastError();
    }
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
        // eight queries per K/V head run as two sets of four (two blocks read the same rows, the second
        // mostly from cache): a block with eight query states needs 256 registers per lane and was slower
        const int kq = q_per_kv == 8 ? 4 : q_per_kv;
        const dim3 grid(n_partials, n_heads, q_per_kv / kq);
        const _Float16* q = reinterpret_cast<const _Float16*>(d_q);
        switch (kq) {
            case 1:
                hipLaunchKernelGGL(k_attn_partial<1>, grid, dim3(256), 0, s, d_rows, pools, layer, n_heads, q, frame_lo,
                                   frame_hi, fpc, n_splits, softmax_scale, d_partial);
                break;
            case 2:
                hipLaunchKernelGGL(k_attn_partial<2>, grid, dim3(256), 0, s, d_rows, pools, layer, n_heads, q, frame_lo,
                                   frame_hi, fpc, n_splits, softmax_scale, d_partial);
                break;
            case 4:
                hipLaunchKernelGGL(k_attn_partial<4>, grid, dim3(256), 0, s, d_rows, pools, layer, n_heads, q, frame_lo,
                                   frame_hi, fpc, n_splits, softmax_scale, d_partial);
                break;
            default:
                return hipErrorInvalidValue;
        }
        if (ev_stop != nullptr && hipEventRecord(ev_stop, s) != hipSuccess) return hipErrorUnknown;
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_attn_merge, dim3(n_heads * q_per_kv), dim3(256), 0, s, d_partial, n_partials, kAttnPartials,
                       d_out, d_lse_or_null);
    return hipGetLastError();
}

}  // namespace sali
