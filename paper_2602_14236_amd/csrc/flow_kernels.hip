// Dense polynomial-expansion optical flow, per-patch motion and the redundancy gate for gfx950.
//
// Temporal Filtering via Optical Flow (Eq. 5, Eq. 6, reuse rule R_frame > theta_R) and
// Implementation Details (Farneback's algorithm, pyramid scale 0.5).  Plain fp32 VALU work on
// small images: no dense contraction here, so no MFMA; the design goal is few launches and no
// spilled intermediates.
//
//   k_expand     pyramid (5x5 binomial [1 4 6 4 1]/16, stride 2; level 0 is gray / 255) and
//                polynomial expansion of up to three levels in ONE launch: 16x16 tiles, the pyramid
//                values a tile needs are rebuilt from the gray image in LDS; separable moments,
//                closed-form solution of the 6-unknown weighted least-squares fit
//   k_pyr_down, k_polyexp   the same per level (pyramid in HBM), used for more than three levels
//   k_flow_iter  one displacement update: per cell of a tile (16x16 or 32x16, by level size) + 5-pixel
//                halo, sample the new frame's expansion bilinearly at x + prior, build A^T A (3 values)
//                and A^T db (2 values) in LDS, separable 11x11 Gaussian aggregation in LDS, 2x2 ridge
//                solve.  The coarse-to-fine transfer (2 * bilinear of the coarser flow) is folded
//                into the first update of a level, so G/h fields never touch HBM.  The gather of
//                the warped expansion is 82 % of a block's time (measured with the wall clock):
//                a chain of dependent HBM round trips, not a throughput limit (vector ALU 78 %,
//                texture addresser 75 % busy at 1920x1080);
//                tiles are handed to the XCDs in contiguous runs so that neighbours share an L2.
//   k_patch_gate per patch RMS flow magnitude (Eq. 5); the last block to finish counts static
//                patches and writes the gate (Eq. 6).  Stand-alone flow call only: the chained
//                step does this inside the pooling kernel.
//
// The batched kernels take the frame as a grid dimension.  All stencils replicate the border.

#include "sali_internal.h"

namespace sali {

namespace {

constexpr int kT = 32;                       // tile side of the expansion kernel
constexpr int kPR = kT + 2 * kPolyN;         // 38

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }
__device__ __forceinline__ float clampf(float v, float lo, float hi) { return fminf(fmaxf(v, lo), hi); }

// Element i of an array whose base is uniform over the wave: base + 32-bit byte offset (an image level
// has fewer than 2^28 pixels, so i * 16 fits), which the hardware adds itself; with 64-bit indices a
// quarter of the gather's vector instructions were address arithmetic.
template <typename V>
__device__ __forceinline__ V ld_at(const V* __restrict__ base, uint32_t i) {
    return *reinterpret_cast<const V*>(reinterpret_cast<const char*>(base) + i * (uint32_t)sizeof(V));
}
__device__ __forceinline__ uint32_t pix(int y, int w, int x) {          // y * w + x, both factors below 2^24
    return __umul24((uint32_t)y, (uint32_t)w) + (uint32_t)x;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// One pyramid level of every frame of the batch (blockIdx.z): level `lvl` of f.pyr[z] from level
// lvl - 1 (from the gray image f.y8[z] for lvl = 1).
__global__ __launch_bounds__(256) void k_pyr_down(PyrBatch f, int from_gray, long long src_off, long long dst_off,
                                                  int sh, int sw, int dh, int dw) {
    const uint8_t* __restrict__ y8 = from_gray ? f.y8[blockIdx.z] : nullptr;
    const float* __restrict__ src = f.pyr[blockIdx.z] + src_off;
    float* __restrict__ dst = f.pyr[blockIdx.z] + dst_off;
    const int x = blockIdx.x * 64 + (threadIdx.x & 63);
    const int y = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (x >= dw || y >= dh) return;
    const float k[5] = {1.0f / 16, 4.0f / 16, 6.0f / 16, 4.0f / 16, 1.0f / 16};
    float acc = 0.0f;
#pragma unroll
    for (int a = -2; a <= 2; ++a) {
        const int yy = clampi(2 * y + a, 0, sh - 1);
        float row = 0.0f;
#pragma unroll
        for (int b = -2; b <= 2; ++b) {
            const int xx = clampi(2 * x + b, 0, sw - 1);
            const float v = y8 != nullptr ? (float)y8[(size_t)yy * sw + xx] / 255.0f : src[(size_t)yy * sw + xx];
            row += k[b + 2] * v;
        }
        acc += k[a + 2] * row;
    }
    dst[(size_t)y * dw + x] = acc;
}

// ---------------------------------------------------------------------------------------------
// Polynomial expansion f(x + d) ~ c + b.d + d^T A d over the 7x7 Gaussian-weighted window.
// With separable symmetric weights (sum 1, second moment m2, fourth moment m4) the normal
// equations decouple:  b = (sx, sy) / m2,  A_xx = (sxx - m2 s0) / (m4 - m2^2),  A_yy likewise,
// A_xy = sxy / (2 m2^2), where s* are the weighted correlations of f with 1, x, y, x^2, y^2, xy.
__global__ __launch_bounds__(256) void k_polyexp(PyrBatch f, LevelGeom g, FlowWeights fw) {
    // blockIdx.y = frame of the batch
    const uint8_t* __restrict__ y8 = f.y8[blockIdx.y];
    const float* __restrict__ pyr = f.pyr[blockIdx.y];
    float4* __restrict__ A_out = f.A[blockIdx.y];
    float* __restrict__ b_out = f.b[blockIdx.y];
    // unpadded rows: the passes that write and read these arrays column-wise address them linearly
    // in the thread index (with a pad of one float, a group of 32 lanes that straddles two rows has
    // two lanes on one bank: 23 % of the kernel's LDS cycles were bank conflicts)
    __shared__ float s_f[kPR][kPR];
    __shared__ float s_v[3][kT][kPR];

    int lvl = 0;
    while (lvl + 1 < g.levels && (int)blockIdx.x >= g.tile_start[lvl + 1]) ++lvl;
    const int t = blockIdx.x - g.tile_start[lvl];
    const int h = g.h[lvl], w = g.w[lvl];
    const int x0 = (t % g.tiles_x[lvl]) * kT, y0 = (t / g.tiles_x[lvl]) * kT;
    const float* src = pyr + g.off[lvl];
    const int tid = threadIdx.x;

    for (int p = tid; p < kPR * kPR; p += 256) {
        const int ry = p / kPR, rx = p % kPR;
        const int gy = clampi(y0 - kPolyN + ry, 0, h - 1), gx = clampi(x0 - kPolyN + rx, 0, w - 1);
        const size_t gi = (size_t)gy * w + gx;
        s_f[ry][rx] = (lvl == 0) ? (float)y8[gi] / 255.0f : src[gi];
    }
    __syncthreads();

    // Out-of-image cells of the region hold the value at the clamped coordinate, which is exactly
    // what a replicate-border stencil centred on an in-image pixel reads.  Vertical moments:
    for (int p = tid; p < kT * kPR; p += 256) {
        const int ty = p / kPR, rx = p % kPR;
        float v0 = 0.0f, v1 = 0.0f, v2 = 0.0f;
#pragma unroll
        for (int k = -kPolyN; k <= kPolyN; ++k) {
            const float f = s_f[ty + kPolyN + k][rx] * fw.poly_g[k + kPolyN];
            v0 += f;
            v1 += f * (float)k;
            v2 += f * (float)(k * k);
        }
        s_v[0][ty][rx] = v0;
        s_v[1][ty][rx] = v1;
        s_v[2][ty][rx] = v2;
    }
    __syncthreads();

    for (int p = tid; p < kT * kT; p += 256) {
        const int ty = p / kT, tx = p % kT;
        const int gy = y0 + ty, gx = x0 + tx;
        if (gy >= h || gx >= w) continue;
        float s0 = 0, sx = 0, sxx = 0, sy = 0, sxy = 0, syy = 0;
#pragma unroll
        for (int k = -kPolyN; k <= kPolyN; ++k) {
            const float gk = fw.poly_g[k + kPolyN];
            const float a0 = s_v[0][ty][tx + kPolyN + k] * gk;
            const float a1 = s_v[1][ty][tx + kPolyN + k] * gk;
            const float a2 = s_v[2][ty][tx + kPolyN + k] * gk;
            s0 += a0;
            sx += a0 * (float)k;
            sxx += a0 * (float)(k * k);
            sy += a1;
            sxy += a1 * (float)k;
            syy += a2;
        }
        const size_t gi = g.off[lvl] + (size_t)gy * w + gx;
        const float axx = (sxx - fw.m2 * s0) * fw.inv_den;
        const float ayy = (syy - fw.m2 * s0) * fw.inv_den;
        const float axy = sxy * fw.inv_2m2sq;
        A_out[gi] = make_float4(axx, axy, ayy, sx * fw.inv_m2);
        b_out[gi] = sy * fw.inv_m2;
    }
}

// ---------------------------------------------------------------------------------------------
// Pyramid + expansion in one launch for up to three levels: a block owns one 16x16 tile of one
// level and rebuilds the pyramid values it needs from the gray image in LDS (level 1 from a 47x47
// gray patch, level 2 from a 47x47 level-1 patch built from a 97x97 gray patch).  This recomputes
// some pyramid pixels but removes two dependent launches and all pyramid traffic.
namespace {
constexpr int kET = 16;                        // tile side
constexpr int kER = kET + 2 * kPolyN;          // 22: region the expansion stencil reads
constexpr int kEP = 2 * (kER - 1) + 5;         // 47: region one level below that feeds it
constexpr int kEQ = 2 * (kEP - 1) + 5;         // 97: region two levels below
// The 47-wide float patch is de-interleaved: even columns from float 24 of a row on, row stride 59, so
// that the stage reading it (22 cells per row) sees addresses linear in its thread index (pyr_level_lds:
// 2 * 59 = 22 mod 32); its writes, one per 25 reads, then see two-way conflicts (even columns at 48 would
// need rows of 75 floats).  The 97-wide gray patch of a level-2 tile stays in bytes, plain layout, rows of
// 112 bytes: the stage that reads it takes 47 cells per row by 48 lanes at a stride of two bytes, so a
// group of 32 lanes reads 16 words (two lanes a word: a broadcast), and the second half of a wave,
// which straddles two cell rows = 2 * 28 words = 24 banks apart, still hits every bank at most once.
constexpr int kEvenP = 24, kEPS = 59;
constexpr int kEQB = 112;
static_assert(kEvenP + (kEP + 1) / 2 <= kEPS && kEvenP >= kEP / 2, "a row holds both halves");
static_assert(kEQB % 4 == 0 && kEQB >= (kEQ + 3) / 4 * 4 && (2 * (kEQB / 4)) % 32 == 24, "byte rows");

// LDS patches that feed a pyramid stage keep the odd columns of a row in its first part and the even
// columns from kEven on (kEven = 0: plain layout): the stage reads columns 2 * cx + {-2..2}, a stride
// of two over the lanes, which in the plain layout puts two lanes on every bank (measured: bank-conflict
// cycles were 45 % of the kernel's LDS cycles); de-interleaved, every tap is a unit-stride read.
template <int kEven>
__device__ __forceinline__ int lds_col(int c) {
    return kEven == 0 ? c : (c & 1 ? 0 : kEven) + (c >> 1);
}

// one level of the 5x5 binomial pyramid, LDS to LDS.  dst cell i (i < kN) stands for the
// coordinate clamp(o_dst + i) of the upper level and reads src cells 2 * that + {-2..2} - o_src
// (o_src is even, so the parity of a tap's column is the parity of the tap).  Threads take the cells in
// row-major order, kLanesPerRow (>= kN) lanes per row; with 2 * kSrcStride = kLanesPerRow (mod 32) the
// address of a tap is thread index + constant, i.e. free of bank conflicts.
template <int kSrcStride, int kSrcEven, int kDstStride, int kDstEven, int kN, int kLanesPerRow>
__device__ __forceinline__ void pyr_level_lds(const float* src, int o_src_y, int o_src_x, float* dst, int o_dst_y,
                                              int o_dst_x, int dh, int dw) {
    static_assert((2 * kSrcStride - kLanesPerRow) % 32 == 0, "tap addresses must be linear in the thread index");
    const float k[5] = {1.0f / 16, 4.0f / 16, 6.0f / 16, 4.0f / 16, 1.0f / 16};
    for (int p = threadIdx.x; p < kN * kLanesPerRow; p += 256) {
        const int ry = p / kLanesPerRow, rx = p % kLanesPerRow;
        if (rx >= kN) continue;
        const int cy = clampi(o_dst_y + ry, 0, dh - 1), cx = clampi(o_dst_x + rx, 0, dw - 1);
        const int sy = 2 * cy - o_src_y, sx = 2 * cx - o_src_x;
        float acc = 0.0f;
#pragma unroll
        for (int a = -2; a <= 2; ++a) {
            float row = 0.0f;
#pragma unroll
            for (int b = -2; b <= 2; ++b) row += k[b + 2] * src[(sy + a) * kSrcStride + lds_col<kSrcEven>(sx + b)];
            acc += k[a + 2] * row;
        }
        dst[ry * kDstStride + lds_col<kDstEven>(rx)] = acc;
    }
}
// Gray patch of kSide x kSide pixels with origin (qy, qx) (coordinates clamped to the image) into LDS
// as gray / 255, row stride kStride, columns laid out by lds_col<kEven>.  All of a thread's loads are
// issued before the first one is used: written as one loop the compiler waits for every byte in turn,
// up to 37 dependent round trips, and next to a kernel that saturates the memory system each of them
// takes microseconds.
template <int kSide, int kStride, int kEven>
__device__ __forceinline__ void load_gray_patch(const uint8_t* __restrict__ y8, int h0, int w0, int qy, int qx,
                                                float* __restrict__ dst) {
    constexpr int kN = (kSide * kSide + 255) / 256;
    uint8_t v[kN];
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        const int p = (int)threadIdx.x + 256 * k;
        const int pp = p < kSide * kSide ? p : 0;
        const int ry = pp / kSide, rx = pp % kSide;
        const int gy = clampi(qy + ry, 0, h0 - 1), gx = clampi(qx + rx, 0, w0 - 1);
        v[k] = y8[(size_t)gy * w0 + gx];
    }
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        const int p = (int)threadIdx.x + 256 * k;
        if (p < kSide * kSide) dst[(p / kSide) * kStride + lds_col<kEven>(p % kSide)] = (float)v[k] / 255.0f;
    }
}

// The 97 x 97 gray patch of a level-2 tile, origin (qy, qx), coordinates clamped to the image, as bytes:
// a thread takes four columns at a time (one 32-bit LDS write; one 32-bit load where the four lie inside the
// image, the compiler is told nothing about its alignment) and has all its loads in flight before the
// first is used.  As floats the patch took 40 KB and the block 52: three blocks per compute unit, also for
// the level-0 and level-1 tiles of the same launch, which need none of it; in bytes the block takes 24 KB.
__device__ __forceinline__ void load_gray_patch_bytes(const uint8_t* __restrict__ y8, int h0, int w0, int qy, int qx,
                                                      uint32_t* __restrict__ dst) {
    constexpr int kQuads = (kEQ + 3) / 4, kItems = kEQ * kQuads, kN = (kItems + 255) / 256;
    uint32_t v[kN];
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        const int p = (int)threadIdx.x + 256 * k;
        const int pp = p < kItems ? p : 0;
        const int ry = pp / kQuads, x = qx + 4 * (pp % kQuads);
        const uint8_t* row = y8 + (size_t)clampi(qy + ry, 0, h0 - 1) * w0;
        if (x >= 0 && x + 3 < w0) {
            __builtin_memcpy(&v[k], row + x, 4);
        } else {
            v[k] = (uint32_t)row[clampi(x, 0, w0 - 1)] | ((uint32_t)row[clampi(x + 1, 0, w0 - 1)] << 8) |
                   ((uint32_t)row[clampi(x + 2, 0, w0 - 1)] << 16) | ((uint32_t)row[clampi(x + 3, 0, w0 - 1)] << 24);
        }
    }
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        const int p = (int)threadIdx.x + 256 * k;
        if (p < kItems) dst[(p / kQuads) * (kEQB / 4) + p % kQuads] = v[k];
    }
}

// First pyramid level of a level-2 tile from the byte patch: the 5x5 binomial sum in integers (weights
// 1 4 6 4 1 squared: at most 256 * 255, exact) and one division by 256 * 255, i.e. the level-1 value of
// gray / 255 rounded once.  Cells and lanes as in pyr_level_lds.
template <int kDstStride, int kDstEven, int kN, int kLanesPerRow>
__device__ __forceinline__ void pyr_level_from_bytes(const uint8_t* src, int o_src_y, int o_src_x, float* dst,
                                                     int o_dst_y, int o_dst_x, int dh, int dw) {
    const uint32_t k[5] = {1u, 4u, 6u, 4u, 1u};
    for (int p = threadIdx.x; p < kN * kLanesPerRow; p += 256) {
        const int ry = p / kLanesPerRow, rx = p % kLanesPerRow;
        if (rx >= kN) continue;
        const int cy = clampi(o_dst_y + ry, 0, dh - 1), cx = clampi(o_dst_x + rx, 0, dw - 1);
        const int sy = 2 * cy - o_src_y, sx = 2 * cx - o_src_x;
        uint32_t acc = 0u;
#pragma unroll
        for (int a = -2; a <= 2; ++a) {
            uint32_t row = 0u;
#pragma unroll
            for (int b = -2; b <= 2; ++b) row += k[b + 2] * (uint32_t)src[(sy + a) * kEQB + sx + b];
            acc += k[a + 2] * row;
        }
        dst[ry * kDstStride + lds_col<kDstEven>(rx)] = (float)acc / 65280.0f;
    }
}

}  // namespace

__global__ __launch_bounds__(256) void k_expand(ExpandBatch f, LevelGeom g, int t1, int t2, int tx0, int tx1, int tx2,
                                                FlowWeights fw) {
    // Work order.  A level-2 tile costs about ten times a level-0 tile (97 x 97 gray pixels, two pyramid
    // stages) and there are sixteen level-0 tiles for each: with the tiles of a frame in level order the
    // heavy ones start last and the launch ends with a few of them on an idle chip (22 us per four
    // 336x336 frames, 10 of them that tail).  So the linear block id is cut into runs, heaviest first,
    // each run over all frames of the batch: level-2 tiles, level-1 tiles, level-0 tiles.
    const int n_frames = (int)gridDim.y;
    const int t3 = (int)gridDim.x;                  // tiles of a frame over all levels
    int idx = (int)blockIdx.x + (int)gridDim.x * (int)blockIdx.y;
    int lvl, t, frame;
    if (idx < n_frames * (t3 - t2)) {
        lvl = 2;
        frame = idx / (t3 - t2);
        t = idx - frame * (t3 - t2);
    } else if ((idx -= n_frames * (t3 - t2)) < n_frames * (t2 - t1)) {
        lvl = 1;
        frame = idx / (t2 - t1);
        t = idx - frame * (t2 - t1);
    } else {
        idx -= n_frames * (t2 - t1);
        lvl = 0;
        frame = idx / t1;
        t = idx - frame * t1;
    }
    const uint8_t* __restrict__ y8 = f.y8[frame];
    float4* __restrict__ A_out = f.A[frame];
    float* __restrict__ b_out = f.b[frame];
    __shared__ uint32_t s_qb[kEQ * (kEQB / 4)];     // gray patch of a level-2 block, bytes
    __shared__ float s_p[kEP * kEPS];               // level-1 patch of a level-2 block; gray patch of a level-1 block
    // unpadded rows: both the pass that writes these arrays and the pass that reads them then see
    // addresses linear in the thread index (the horizontal pass pairs rows eight apart, see below)
    __shared__ float s_f[kER][kER];
    // the vertical moments reuse the 47-wide patch's memory: every path has a barrier between its last
    // read of s_p and the pass that writes them
    float (*s_v)[kET][kER] = reinterpret_cast<float (*)[kET][kER]>(s_p);
    static_assert(3 * kET * kER <= kEP * kEPS, "moments fit into the 47-wide patch");

    const int tiles_x = lvl == 0 ? tx0 : (lvl == 1 ? tx1 : tx2);
    const int h = g.h[lvl], w = g.w[lvl];
    const int x0 = (t % tiles_x) * kET, y0 = (t / tiles_x) * kET;
    const int oy = y0 - kPolyN, ox = x0 - kPolyN;   // origin of s_f in this level's coordinates
    const int tid = threadIdx.x;
    const int h0 = g.h[0], w0 = g.w[0];

    if (lvl == 0) {
        load_gray_patch<kER, kER, 0>(y8, h, w, oy, ox, &s_f[0][0]);
    } else if (lvl == 1) {
        const int qy = 2 * oy - 2, qx = 2 * ox - 2;              // origin of the gray patch (47 x 47)
        load_gray_patch<kEP, kEPS, kEvenP>(y8, h0, w0, qy, qx, s_p);
        __syncthreads();
        pyr_level_lds<kEPS, kEvenP, kER, 0, kER, kER>(s_p, qy, qx, &s_f[0][0], oy, ox, h, w);
    } else {
        const int h1 = g.h[1], w1 = g.w[1];
        const int py = 2 * oy - 2, px = 2 * ox - 2;              // origin of the level-1 patch (47 x 47)
        const int qy = 2 * py - 2, qx = 2 * px - 2;              // origin of the gray patch (97 x 97)
        load_gray_patch_bytes(y8, h0, w0, qy, qx, s_qb);
        __syncthreads();
        pyr_level_from_bytes<kEPS, kEvenP, kEP, kEP + 1>(reinterpret_cast<const uint8_t*>(s_qb), qy, qx, s_p, py, px, h1,
                                                         w1);
        __syncthreads();
        pyr_level_lds<kEPS, kEvenP, kER, 0, kER, kER>(s_p, py, px, &s_f[0][0], oy, ox, h, w);
    }
    __syncthreads();

    // vertical moments, then horizontal moments and the closed-form fit (as in k_polyexp)
    for (int p = tid; p < kET * kER; p += 256) {
        const int ty = p / kER, rx = p % kER;
        float v0 = 0.0f, v1 = 0.0f, v2 = 0.0f;
#pragma unroll
        for (int k = -kPolyN; k <= kPolyN; ++k) {
            const float f = s_f[ty + kPolyN + k][rx] * fw.poly_g[k + kPolyN];
            v0 += f;
            v1 += f * (float)k;
            v2 += f * (float)(k * k);
        }
        s_v[0][ty][rx] = v0;
        s_v[1][ty][rx] = v1;
        s_v[2][ty][rx] = v2;
    }
    __syncthreads();
    {
        // a group of 32 lanes takes the rows r and r + 8 (16 lanes each): 8 rows of 22 floats are 176 =
        // 16 (mod 32) floats apart, so the two rows lie on disjoint banks
        const int half = tid / kET, tx = tid % kET;
        const int ty = (half >> 1) + 8 * (half & 1);
        const int gy = y0 + ty, gx = x0 + tx;
        if (gy < h && gx < w) {
            float s0 = 0, sx = 0, sxx = 0, sy = 0, sxy = 0, syy = 0;
#pragma unroll
            for (int k = -kPolyN; k <= kPolyN; ++k) {
                const float gk = fw.poly_g[k + kPolyN];
                const float a0 = s_v[0][ty][tx + kPolyN + k] * gk;
                const float a1 = s_v[1][ty][tx + kPolyN + k] * gk;
                const float a2 = s_v[2][ty][tx + kPolyN + k] * gk;
                s0 += a0;
                sx += a0 * (float)k;
                sxx += a0 * (float)(k * k);
                sy += a1;
                sxy += a1 * (float)k;
                syy += a2;
            }
            const size_t gi = g.off[lvl] + (size_t)gy * w + gx;
            A_out[gi] = make_float4((sxx - fw.m2 * s0) * fw.inv_den, sxy * fw.inv_2m2sq, (syy - fw.m2 * s0) * fw.inv_den,
                                    sx * fw.inv_m2);
            b_out[gi] = sy * fw.inv_m2;
        }
    }
}

// ---------------------------------------------------------------------------------------------
namespace {

// bilinear sample of a float2 field at real (y, x), coordinates clamped to the image
__device__ __forceinline__ float2 bilerp2(const float2* __restrict__ f, int h, int w, float y, float x) {
    y = clampf(y, 0.0f, (float)(h - 1));
    x = clampf(x, 0.0f, (float)(w - 1));
    const float fy0 = floorf(y), fx0 = floorf(x);
    const int y0 = (int)fy0, x0 = (int)fx0;
    const int y1 = min(y0 + 1, h - 1), x1 = min(x0 + 1, w - 1);
    const float wy = y - fy0, wx = x - fx0;
    const float2 a = ld_at(f, pix(y0, w, x0)), b = ld_at(f, pix(y0, w, x1));
    const float2 c = ld_at(f, pix(y1, w, x0)), d = ld_at(f, pix(y1, w, x1));
    const float tx = a.x * (1.0f - wx) + b.x * wx, ty = a.y * (1.0f - wx) + b.y * wx;
    const float bx = c.x * (1.0f - wx) + d.x * wx, by = c.y * (1.0f - wx) + d.y * wx;
    return make_float2(tx * (1.0f - wy) + bx * wy, ty * (1.0f - wy) + by * wy);
}

// prior displacement of a pixel: 0 (coarsest level), 2 * bilinear(coarser flow; y/2, x/2) for
// the first update of a finer level, or the previous update's result
__device__ __forceinline__ float2 prior_at(const float2* __restrict__ d_in, int mode, int gy, int gx, int w, int ch,
                                           int cw) {
    if (mode == 0) return make_float2(0.0f, 0.0f);
    if (mode == 1) {
        const float2 c = bilerp2(d_in, ch, cw, 0.5f * (float)gy, 0.5f * (float)gx);
        return make_float2(2.0f * c.x, 2.0f * c.y);
    }
    return ld_at(d_in, pix(gy, w, gx));
}

// Row and column of item p of a window pass over n_rows rows of TX outputs; false = an idle lane.
// TX = 32: row-major.  TX = 16: the 32 lanes of a group take rows r and r + 8 (first the whole blocks of 16
// rows: groups 0..7 take rows (0,8) .. (7,15); of the rest, n_rows - 16 k <= 15 rows, those that have a
// partner eight further on are paired, the others get a group of their own with its upper half idle).
template <int TX>
__device__ __forceinline__ bool window_item(int p, int n_rows, int& row, int& col) {
    if constexpr (TX == 16) {
        const int g = p >> 5, half = (p >> 4) & 1;
        col = p & 15;
        const int full = n_rows / 16, base = 16 * full;
        if (g < 8 * full) {
            row = (g >> 3) * 16 + (g & 7) + 8 * half;
            return true;
        }
        const int rest = n_rows - base, gg = g - 8 * full, npair = rest > 8 ? rest - 8 : 0;
        if (gg < npair) {
            row = base + gg + 8 * half;
            return true;
        }
        row = base + npair + (gg - npair);
        return half == 0 && row < base + (rest > 8 ? 8 : rest);
    } else {
        row = p / TX;
        col = p % TX;
        return row < n_rows;
    }
}
// items (lanes, idle ones included) of such a pass
template <int TX>
constexpr int window_items(int n_rows) {
    if (TX != 16) return n_rows * TX;
    const int rest = n_rows % 16, npair = rest > 8 ? rest - 8 : 0;
    return 32 * (8 * (n_rows / 16) + npair + ((rest > 8 ? 8 : rest) - npair));
}

}  // namespace

// TX x TY = tile, NT = threads of the block.
template <int TX, int TY, int NT>
__global__ __launch_bounds__(NT) void k_flow_iter(FlowBatch f, long long level_off, int h, int w, int ch, int cw,
                                                  int prior_mode, FlowWeights fw) {
    // blk.z = frame of the batch, (blk.x, blk.y) = tile
    const BlockId blk = xcd_block_id();
    const float4* __restrict__ A1 = f.A1[blk.z] + level_off;
    const float* __restrict__ b1 = f.b1[blk.z] + level_off;
    const float4* __restrict__ A2 = f.A2[blk.z] + level_off;
    const float* __restrict__ b2 = f.b2[blk.z] + level_off;
    const float2* __restrict__ d_in = f.d_in[blk.z];
    float2* __restrict__ d_out = f.d_out[blk.z];
    constexpr int RX = TX + 2 * kWinR, RY = TY + 2 * kWinR;
    // Row stride of the per-cell terms.  A group of 32 lanes of a window pass reads one row of a 32-wide
    // tile but two rows (16 lanes each) of a 16-wide one, which must not share banks: their distance has
    // to be 16 mod 32 floats.  With adjacent rows that takes a stride of 48 floats for 26 cells (25 KB a
    // block, five blocks per compute unit; RX + 1 = 27 spent 37 % of the LDS cycles on bank conflicts).
    // Instead the two rows of a group are eight apart (window_item) and the rows are unpadded: 8 * 26 = 16
    // mod 32; the pass that writes the terms then sees addresses linear in the thread index, and a block
    // takes 16 KB, so that eight blocks fill every wave slot of a compute unit.
    constexpr int RXS = TX == 16 ? RX : RX + 1;
    static_assert(TX != 16 || (8 * RXS) % 32 == 16, "rows eight apart sit 16 banks apart");
    __shared__ float s_in[5][RY][RXS];
    __shared__ float2 s_dp[TY][TX];          // prior of the tile's own pixels, for the solve

    const int tid = threadIdx.x;
    const int x0 = blk.x * TX, y0 = blk.y * TY;

    // per-cell A^T A and A^T db at the clamped coordinate of the cell
#pragma unroll 2
    for (int p = tid; p < RX * RY; p += NT) {
        const int ry = p / RX, rx = p % RX;
        const int gy = clampi(y0 - kWinR + ry, 0, h - 1), gx = clampi(x0 - kWinR + rx, 0, w - 1);
        const uint32_t gi = pix(gy, w, gx);
        const float2 dp = prior_at(d_in, prior_mode, gy, gx, w, ch, cw);
        if (ry >= kWinR && ry < kWinR + TY && rx >= kWinR && rx < kWinR + TX) s_dp[ry - kWinR][rx - kWinR] = dp;
        const float4 a1 = ld_at(A1, gi);
        const float2 bb1 = make_float2(a1.w, ld_at(b1, gi));
        // sample the new frame's expansion at x + prior
        const float sy = clampf((float)gy + dp.y, 0.0f, (float)(h - 1));
        const float sx = clampf((float)gx + dp.x, 0.0f, (float)(w - 1));
        const float fy0 = floorf(sy), fx0 = floorf(sx);
        const int iy0 = (int)fy0, ix0 = (int)fx0;
        const int iy1 = min(iy0 + 1, h - 1), ix1 = min(ix0 + 1, w - 1);
        const float wy = sy - fy0, wx = sx - fx0;
        const uint32_t i00 = pix(iy0, w, ix0), i10 = pix(iy1, w, ix0);
        const uint32_t i01 = i00 + (uint32_t)(ix1 - ix0), i11 = i10 + (uint32_t)(ix1 - ix0);
        const float4 a00 = ld_at(A2, i00), a01 = ld_at(A2, i01), a10 = ld_at(A2, i10), a11 = ld_at(A2, i11);
        const float2 c00 = make_float2(a00.w, ld_at(b2, i00)), c01 = make_float2(a01.w, ld_at(b2, i01));
        const float2 c10 = make_float2(a10.w, ld_at(b2, i10)), c11 = make_float2(a11.w, ld_at(b2, i11));
        const float w00 = (1.0f - wx) * (1.0f - wy), w01 = wx * (1.0f - wy), w10 = (1.0f - wx) * wy, w11 = wx * wy;
        const float a2xx = a00.x * w00 + a01.x * w01 + a10.x * w10 + a11.x * w11;
        const float a2xy = a00.y * w00 + a01.y * w01 + a10.y * w10 + a11.y * w11;
        const float a2yy = a00.z * w00 + a01.z * w01 + a10.z * w10 + a11.z * w11;
        const float b2x = c00.x * w00 + c01.x * w01 + c10.x * w10 + c11.x * w11;
        const float b2y = c00.y * w00 + c01.y * w01 + c10.y * w10 + c11.y * w11;
        const float axx = 0.5f * (a1.x + a2xx), axy = 0.5f * (a1.y + a2xy), ayy = 0.5f * (a1.z + a2yy);
        const float dbx = -0.5f * (b2x - bb1.x) + axx * dp.x + axy * dp.y;
        const float dby = -0.5f * (b2y - bb1.y) + axy * dp.x + ayy * dp.y;
        s_in[0][ry][rx] = axx * axx + axy * axy;
        s_in[1][ry][rx] = axy * (axx + ayy);
        s_in[2][ry][rx] = axy * axy + ayy * ayy;
        s_in[3][ry][rx] = axx * dbx + axy * dby;
        s_in[4][ry][rx] = axy * dbx + ayy * dby;
    }
    __syncthreads();

    {
        // Row pass of the separable Gaussian window, in place: every thread keeps the sums of its (at most
        // kRowItems) outputs in registers until all taps of all threads are read, then writes them over the
        // terms at [ry][tx].  A second array for the row sums would cost 17 KB (32x16 tile): with it three
        // blocks fit a compute unit, without it four, and next to the K/V kernels, where a block spends its
        // time waiting for memory, the blocks in flight are what sets the kernel's speed.
        constexpr int kRowItems = (window_items<TX>(RY) + NT - 1) / NT;
        float racc[kRowItems][5];
#pragma unroll
        for (int q = 0; q < kRowItems; ++q) {
            const int p = tid + q * NT;
            int ry, tx;
            const bool mine = window_item<TX>(p, RY, ry, tx);
#pragma unroll
            for (int c = 0; c < 5; ++c) racc[q][c] = 0.0f;
            if (mine) {
#pragma unroll
                for (int k = 0; k <= 2 * kWinR; ++k) {
                    const float wk = fw.win_g[k];
#pragma unroll
                    for (int c = 0; c < 5; ++c) racc[q][c] += wk * s_in[c][ry][tx + k];
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kRowItems; ++q) {
            const int p = tid + q * NT;
            int ry, tx;
            if (window_item<TX>(p, RY, ry, tx)) {
#pragma unroll
                for (int c = 0; c < 5; ++c) s_in[c][ry][tx] = racc[q][c];
            }
        }
        __syncthreads();
    }

    // column pass + ridge solve
    for (int p = tid; p < TX * TY; p += NT) {
        int ty, tx;
        window_item<TX>(p, TY, ty, tx);
        const int gy = y0 + ty, gx = x0 + tx;
        if (gy >= h || gx >= w) continue;
        float acc[5] = {0, 0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k <= 2 * kWinR; ++k) {
            const float wk = fw.win_g[k];
#pragma unroll
            for (int c = 0; c < 5; ++c) acc[c] += wk * s_in[c][ty + k][tx];
        }
        const float2 dp = s_dp[ty][tx];
        const float lam = kLamAbs + kLamRel * 0.5f * (acc[0] + acc[2]);
        const float m11 = acc[0] + lam, m22 = acc[2] + lam, m12 = acc[1];
        const float r1 = acc[3] + lam * dp.x, r2 = acc[4] + lam * dp.y;
        const float det = m11 * m22 - m12 * m12;
        *reinterpret_cast<float2*>(reinterpret_cast<char*>(d_out) + pix(gy, w, gx) * 8u) =
            make_float2((m22 * r1 - m12 * r2) / det, (m11 * r2 - m12 * r1) / det);
    }
}

// ---------------------------------------------------------------------------------------------
// Eq. 5 / Eq. 6.  One wave per patch, four patches per block of 256 threads (small blocks find
// room next to other streams' kernels); the last block to finish evaluates the gate.
constexpr int kGateBlocks = kTokens / 4;

__global__ __launch_bounds__(256) void k_patch_gate(const float2* __restrict__ flow, int h, int w, float tau_t,
                                                    float theta_r, float* dp_out, sali_gate* gate,
                                                    uint32_t* done_counter, float* __restrict__ flow_uv) {
    __shared__ int s_cnt[4];
    __shared__ int s_last;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int token = blockIdx.x * 4 + wave;
    const int pr = token / kGrid, pc = token % kGrid;
    const int ya = (pr * h) / kGrid, yb = ((pr + 1) * h) / kGrid;
    const int xa = (pc * w) / kGrid, xb = ((pc + 1) * w) / kGrid;
    const int pw = xb - xa, area = pw * (yb - ya);
    float acc = 0.0f;
    for (int p = lane; p < area; p += 64) {
        const int y = ya + p / pw, x = xa + p % pw;
        const float2 d = flow[(size_t)y * w + x];
        acc += d.x * d.x + d.y * d.y;
        if (flow_uv != nullptr) {
            flow_uv[(size_t)y * w + x] = d.x;
            flow_uv[(size_t)h * w + (size_t)y * w + x] = d.y;
        }
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off);
    if (lane == 0)
        __hip_atomic_store(dp_out + token, sqrtf(acc / (float)area), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        const uint32_t prev = atomicAdd(done_counter, 1u);
        s_last = (prev == (uint32_t)(kGateBlocks - 1)) ? 1 : 0;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    int n = 0;
    for (int i = threadIdx.x; i < kTokens; i += 256) {
        const float v = __hip_atomic_load(dp_out + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        n += (v < tau_t) ? 1 : 0;
    }
    for (int off = 32; off > 0; off >>= 1) n += __shfl_down(n, off);
    if (lane == 0) s_cnt[wave] = n;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int n_static = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
        const float r = (float)n_static / (float)kTokens;
        sali_gate gt;
        gt.n_static = n_static;
        gt.r_frame = r;
        gt.redundant = (r > theta_r) ? 1 : 0;
        gt.reserved = 0;
        *gate = gt;
        *done_counter = 0u;         // ready for the next launch
    }
}

// ---------------------------------------------------------------------------------------------
hipError_t launch_pyr_down(const PyrBatch& f, int n, const LevelGeom& g, int lvl, hipStream_t s) {
    dim3 grid((g.w[lvl] + 63) / 64, (g.h[lvl] + 3) / 4, n);
    hipLaunchKernelGGL(k_pyr_down, grid, dim3(256), 0, s, f, lvl == 1 ? 1 : 0, (long long)g.off[lvl - 1],
                       (long long)g.off[lvl], g.h[lvl - 1], g.w[lvl - 1], g.h[lvl], g.w[lvl]);
    return hipGetLastError();
}

hipError_t launch_polyexp(const PyrBatch& f, int n, LevelGeom g, FlowWeights fw, hipStream_t s) {
    hipLaunchKernelGGL(k_polyexp, dim3(g.tile_start[g.levels], n), dim3(256), 0, s, f, g, fw);
    return hipGetLastError();
}

hipError_t launch_expand(const ExpandBatch& f, int n, LevelGeom g, FlowWeights fw, hipStream_t s) {
    // up to three levels, 16x16 tiles, one launch
    int tx[3] = {1, 1, 1}, start[4] = {0, 0, 0, 0};
    for (int l = 0; l < 3; ++l) {
        int tiles = 0;
        if (l < g.levels) {
            tx[l] = (g.w[l] + kET - 1) / kET;
            tiles = tx[l] * ((g.h[l] + kET - 1) / kET);
        }
        start[l + 1] = start[l] + tiles;
    }
    hipLaunchKernelGGL(k_expand, dim3(start[3], n), dim3(256), 0, s, f, g, start[1], start[2], tx[0], tx[1], tx[2], fw);
    return hipGetLastError();
}

hipError_t launch_flow_iter(const FlowBatch& f, int n, int64_t level_off, int h, int w, int ch, int cw,
                            int prior_mode, FlowWeights fw, hipStream_t s) {
    // Tile and block by level size:
    //   below 40 000 pixels   16x16, 256 threads   (16 KB of LDS: eight blocks per compute unit)
    //   above                 32x16, 512 threads   (26 KB: four blocks; 2.1 instead of 2.6 halo cells per output)
    // A block is a chain of dependent HBM round trips (prior -> warped gather, once per cell a thread
    // owns); with twice the threads a thread owns about two cells, taken together.  Both shapes fill every
    // wave slot of a compute unit, which is what counts next to the K/V kernels, where a block mostly waits
    // for memory.  A 32x32 tile on 1024 threads (1.7 halo cells per output, two blocks per compute unit,
    // 64 registers) was used from 150 000 pixels up until the row pass went in place: alone on the GPU it
    // is 1.5 % faster at 1920x1080 (235 against 239 us per frame), inside the pipeline 2 - 3 % slower
    // (1080p 3 090 -> 3 160 frames/s, 640x360 32 150 -> 33 100): a block of 1024 threads needs sixteen free
    // wave slots on one compute unit at once.  The same tile on 512 threads (84 registers, three blocks) is
    // slower everywhere; 22x22 (one thread per cell), 64x16 and 32x16 on 1024 threads are slower as well.
    const long long px = (long long)h * w;
#define SALI_FLOW_LAUNCH(TX, TY, NT)                                                                         \
    hipLaunchKernelGGL((k_flow_iter<TX, TY, NT>), dim3((w + TX - 1) / TX, (h + TY - 1) / TY, n), dim3(NT), 0, \
                       s, f, (long long)level_off, h, w, ch, cw, prior_mode, fw)
    if (px >= 40000) SALI_FLOW_LAUNCH(32, 16, 512);
    else SALI_FLOW_LAUNCH(16, 16, 256);
#undef SALI_FLOW_LAUNCH
    return hipGetLastError();
}

hipError_t launch_patch_gate(const float2* d_flow, int h, int w, float tau_t, float theta_r, float* d_dp,
                             sali_gate* d_gate, uint32_t* d_done_counter, float* d_flow_uv_or_null, hipStream_t s) {
    hipLaunchKernelGGL(k_patch_gate, dim3(kGateBlocks), dim3(256), 0, s, d_flow, h, w, tau_t, theta_r, d_dp, d_gate,
                       d_done_counter, d_flow_uv_or_null);
    return hipGetLastError();
}

}  // namespace sali
