// Saliency map (Canny edges + LAB colour variance) and patch pooling for gfx950.
//
// Spatial Filtering via Saliency-Guided Quantization (saliency map S, Eq. 7) and
// Implementation Details (Canny edge detection combined with adaptive thresholding on the
// local colour variance in LAB).  Everything here is integer arithmetic, so scores are exact.
//
//   k_prep   one pass over the RGB frame, 32x32 tiles with a 4-pixel halo staged in LDS (colour
//            tables held in LDS too):
//            gray -> 5x5 binomial blur -> Sobel -> squared magnitude -> non-maximum suppression
//            -> weak/strong class, and RGB -> 8-bit LAB -> 5x5 variance sum V, plus the frame
//            sum of V (one 64-bit atomic per block).  Also emits the gray image for the flow.
//            8-connected hysteresis is a lock-free union-find over weak/strong pixels.  A
//            pixel's key is its index with bit 31 set for weak pixels; links always point to
//            the smaller key, so the root of a component is a strong pixel iff it has one.
//            k_prep labels the components of its own tile in LDS (label equivalence, no
//            global traffic) and writes each pixel's link to its tile-local root.
//   k_union  joins components across tile borders with global atomics (border pixels only).
//   k_pool   per patch: E = edge pixel whose root is strong, C = V above the frame mean and
//            above a floor; q = sum(E + C); score = floor(q * 2^15 / |P|) / 65536.  In the
//            chained step it also reduces the flow field to the patch's motion (Eq. 5).
//   k_pool_tail  one block per frame: the gate (Eq. 6) and the ranking of the frame's tokens; the
//            last of them to finish writes the frame-table rows in video order.
//
// Every kernel takes the frame as a grid dimension (per-frame pointers in a by-value struct): one
// small frame cannot fill 256 compute units.
//
// All stencils replicate the border; non-maximum suppression treats out-of-image neighbours
// as magnitude 0.

#include "sali_internal.h"
#include "hysteresis.h"
#include "tier_body.h"

namespace sali {

namespace {

constexpr int kHalo = 4;
constexpr int kReg = kTile + 2 * kHalo;        // 40: gray region
constexpr int kRegB = kTile + 4;               // 36: blur / LAB region (halo 2)
constexpr int kRegM = kTile + 2;               // 34: gradient-magnitude region (halo 1)

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }


}  // namespace

// gray only, blockIdx.y = frame of the batch: what the flow needs of a frame.  The rest of the spatial
// filter waits until the reuse rule has spoken.  Sixteen pixels per thread (48 bytes in, 16 out) where
// the caller's image is 16-byte aligned, else pixel by pixel.
__device__ __forceinline__ uint32_t gray_of(uint32_t r, uint32_t g, uint32_t b) {
    return (77u * r + 150u * g + 29u * b + 128u) >> 8;
}

__global__ __launch_bounds__(256) void k_gray(PrepBatch f, int n) {
    const uint8_t* __restrict__ rgb = f.rgb[blockIdx.y];
    uint8_t* __restrict__ y8 = f.y8[blockIdx.y];
    const int i0 = (blockIdx.x * 256 + threadIdx.x) * 16;
    if (i0 >= n) return;
    if (i0 + 16 <= n && (reinterpret_cast<uintptr_t>(rgb) & 15u) == 0) {
        const uint4* src = reinterpret_cast<const uint4*>(rgb + (size_t)i0 * 3);
        const uint4 a = src[0], b = src[1], c = src[2];
        const uint32_t in[12] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w, c.x, c.y, c.z, c.w};
        uint32_t out[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {           // four pixels = three words: RGBR GBRG BRGB
            const uint32_t w0 = in[3 * q], w1 = in[3 * q + 1], w2 = in[3 * q + 2];
            const uint32_t g0 = gray_of(w0 & 0xFF, (w0 >> 8) & 0xFF, (w0 >> 16) & 0xFF);
            const uint32_t g1 = gray_of(w0 >> 24, w1 & 0xFF, (w1 >> 8) & 0xFF);
            const uint32_t g2 = gray_of((w1 >> 16) & 0xFF, w1 >> 24, w2 & 0xFF);
            const uint32_t g3 = gray_of((w2 >> 8) & 0xFF, (w2 >> 16) & 0xFF, w2 >> 24);
            out[q] = g0 | (g1 << 8) | (g2 << 16) | (g3 << 24);
        }
        *reinterpret_cast<uint4*>(y8 + i0) = make_uint4(out[0], out[1], out[2], out[3]);   // lane scratch: 256-byte aligned
        return;
    }
    for (int i = i0; i < n && i < i0 + 16; ++i) {
        const uint8_t* px = rgb + (size_t)i * 3;
        y8[i] = (uint8_t)gray_of(px[0], px[1], px[2]);
    }
}

// #{dP_i < tau_t} over the thread's share of one image's 576 patch motions (block of 256 threads); the
// loads are independent and issued together
__device__ __forceinline__ int count_static(const float* dp, float tau_t) {
    float v[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const int i = (int)threadIdx.x + 256 * k;
        v[k] = i < kTokens ? __hip_atomic_load(dp + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : tau_t;
    }
    return (v[0] < tau_t ? 1 : 0) + (v[1] < tau_t ? 1 : 0) + (v[2] < tau_t ? 1 : 0);
}

// Eq. 6 and the reuse rule for frame b of a launch, evaluated by a whole block of 256 threads from the
// per-patch motions that an earlier kernel left (dp[b] NULL: no predecessor, never redundant): the
// kernels of the spatial filter ask this first and leave at once for a redundant frame (Algorithm 1
// skips its saliency).  Same counts and the same fp32 quotient as the tail kernel that writes the gate,
// so all of them take the same decision.  s_cnt: four ints of LDS.
__device__ __forceinline__ bool frame_redundant(const float* const* dp, int b, const GateParams& gp, int* s_cnt) {
    const int b0 = b - b % gp.tiles;
    if (dp[b0] == nullptr) return false;
    int n = 0;
    for (int j = 0; j < gp.tiles; ++j) n += count_static(dp[b0 + j], gp.tau_t);
    for (int off = 32; off > 0; off >>= 1) n += __shfl_down(n, off);
    if ((threadIdx.x & 63) == 0) s_cnt[threadIdx.x >> 6] = n;
    __syncthreads();
    const int n_static = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
    __syncthreads();
    return (float)n_static / (float)(kTokens * gp.tiles) > gp.theta_r;
}

// 256 threads per 32x32 tile, four output pixels per thread (pixel p = tid + 256 q sits in tile
// row p / 32, so a wave always holds two complete tile rows).  Workgroups are kept this small so
// that they find room on compute units that a bandwidth kernel of another stream keeps busy.
constexpr int kPrepThreads = 256;
constexpr int kPrepPx = kTile * kTile / kPrepThreads;                          // 4
constexpr int kPrepCells = (kReg * kReg + kPrepThreads - 1) / kPrepThreads;   // 7

__global__ __launch_bounds__(kPrepThreads) void k_prep(PrepBatch f, int h, int w, GateParams gp,
                                                       const uint32_t* __restrict__ lut_words, int lo2, int hi2) {
    // blockIdx.z = frame of the batch
    const uint8_t* __restrict__ rgb = f.rgb[blockIdx.z];
    uint8_t* __restrict__ cls_out = f.cls[blockIdx.z];
    uint32_t* __restrict__ var_out = f.var[blockIdx.z];
    uint32_t* __restrict__ parent_out = f.parent[blockIdx.z];
    unsigned long long* msum_acc = f.msum_acc[blockIdx.z];
    unsigned long long* msum_clear = f.msum_clear[blockIdx.z];
    __shared__ uint32_t s_lut[(256 + 4096) / 2];          // lin[256] then fl[4096], 16-bit entries
    __shared__ uint8_t s_y[kReg][kReg];
    __shared__ uint8_t s_b[kRegB][kRegB];
    __shared__ int s_m2[kRegM][kRegM];
    __shared__ __align__(16) uint8_t s_lab[3][kRegB][kRegB];     // read as 32-bit words by the variance stage
    __shared__ unsigned long long s_sum[kPrepThreads / 64];
    __shared__ uint32_t s_lbl[kTile * kTile];             // tile-local union-find links, key = local index | weak bit
    __shared__ uint8_t s_cls[kTile][kTile];

    const int tid = threadIdx.x;
    const int x0 = blockIdx.x * kTile, y0 = blockIdx.y * kTile;
    const uint16_t* s_lin = reinterpret_cast<const uint16_t*>(s_lut);
    const uint16_t* s_fl = s_lin + 256;

    if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0 && msum_clear != nullptr) *msum_clear = 0ull;

    // stage 1a: RGB of the 40x40 region (clamped coordinates).  The loads are issued before the reuse
    // rule is looked at, so that its memory round trip and theirs overlap: most frames are not redundant.
    uint32_t crgb[kPrepCells];
#pragma unroll
    for (int k = 0; k < kPrepCells; ++k) {
        const int p = tid + k * kPrepThreads;
        crgb[k] = 0u;
        if (p < kReg * kReg) {
            const int ry = p / kReg, rx = p % kReg;
            const int gy = clampi(y0 - kHalo + ry, 0, h - 1), gx = clampi(x0 - kHalo + rx, 0, w - 1);
            const uint8_t* px = rgb + ((size_t)gy * w + gx) * 3;
            const uint32_t r = px[0], g = px[1], b = px[2];
            crgb[k] = r | (g << 8) | (b << 16);
        }
    }
    {
        // no saliency for a redundant frame; the frame's first block leaves the decision for the kernels
        // after this one, whose blocks are too small to count 576 patches each
        __shared__ int s_gate[4];
        const bool skip = frame_redundant(f.dp, blockIdx.z, gp, s_gate);
        if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) *f.skip[blockIdx.z] = skip ? 1u : 0u;
        if (skip) return;
    }
    // colour tables -> LDS, gray of the region
    for (int i = tid; i < (256 + 4096) / 2; i += kPrepThreads) s_lut[i] = lut_words[i];
#pragma unroll
    for (int k = 0; k < kPrepCells; ++k) {
        const int p = tid + k * kPrepThreads;
        if (p < kReg * kReg) {
            const uint32_t r = crgb[k] & 0xFF, g = (crgb[k] >> 8) & 0xFF, b = crgb[k] >> 16;
            s_y[p / kReg][p % kReg] = (uint8_t)((77 * r + 150 * g + 29 * b + 128) >> 8);
        }
    }
    __syncthreads();

    // stage 1b: 8-bit LAB of the 36x36 region through the LDS tables
#pragma unroll
    for (int k = 0; k < kPrepCells; ++k) {
        const int p = tid + k * kPrepThreads;
        if (p >= kReg * kReg) continue;
        const int ry = p / kReg, rx = p % kReg;
        if (ry < 2 || ry >= kReg - 2 || rx < 2 || rx >= kReg - 2) continue;
        const int lr = s_lin[crgb[k] & 0xFF], lg = s_lin[(crgb[k] >> 8) & 0xFF], lb = s_lin[(crgb[k] >> 16) & 0xFF];
        const int tx = (1777 * lr + 1541 * lg + 778 * lb + 2048) >> 12;
        const int ty = (871 * lr + 2929 * lg + 296 * lb + 2048) >> 12;
        const int tz = (73 * lr + 448 * lg + 3575 * lb + 2048) >> 12;
        const int fx = s_fl[tx], fy = s_fl[ty], fz = s_fl[tz];
        s_lab[0][ry - 2][rx - 2] = (uint8_t)clampi(((116 * fy - 524288) * 255 + 1638400) / 3276800, 0, 255);
        s_lab[1][ry - 2][rx - 2] = (uint8_t)clampi((500 * (fx - fy) + 4194304 + 16384) >> 15, 0, 255);
        s_lab[2][ry - 2][rx - 2] = (uint8_t)clampi((200 * (fy - fz) + 4194304 + 16384) >> 15, 0, 255);
    }

    const int tx = tid % kTile;
    const int gx = x0 + tx;

    // Region arrays are indexed by (image coordinate - region origin).  A stage evaluates its
    // stencil at the CLAMPED image coordinate c of each region cell and reads its input at
    // clamp(c + offset); both stay inside the previous stage's region.
    const int oy_y = y0 - kHalo, ox_y = x0 - kHalo;      // origin of s_y
    const int oy_b = y0 - 2, ox_b = x0 - 2;              // origin of s_b / s_lab
    const int oy_m = y0 - 1, ox_m = x0 - 1;              // origin of s_m2

    // stage 2: 5x5 binomial blur, (sum + 128) >> 8
    for (int p = tid; p < kRegB * kRegB; p += kPrepThreads) {
        const int ry = p / kRegB, rx = p % kRegB;
        const int cy = clampi(oy_b + ry, 0, h - 1), cx = clampi(ox_b + rx, 0, w - 1);
        const int kw[5] = {1, 4, 6, 4, 1};
        int acc = 0;
#pragma unroll
        for (int a = -2; a <= 2; ++a) {
            const int yy = clampi(cy + a, 0, h - 1) - oy_y;
            int rowacc = 0;
#pragma unroll
            for (int b = -2; b <= 2; ++b) {
                const int xx = clampi(cx + b, 0, w - 1) - ox_y;
                rowacc += kw[b + 2] * s_y[yy][xx];
            }
            acc += kw[a + 2] * rowacc;
        }
        s_b[ry][rx] = (uint8_t)((acc + 128) >> 8);
    }
    __syncthreads();

    // stage 3: Sobel squared magnitude on the 34x34 region; cells outside the image hold 0
    // (that is what non-maximum suppression wants to see there)
    for (int p = tid; p < kRegM * kRegM; p += kPrepThreads) {
        const int ry = p / kRegM, rx = p % kRegM;
        const int my = oy_m + ry, mx = ox_m + rx;
        int m2 = 0;
        if (my >= 0 && my < h && mx >= 0 && mx < w) {
            const int ym = clampi(my - 1, 0, h - 1) - oy_b, yc = my - oy_b, yp = clampi(my + 1, 0, h - 1) - oy_b;
            const int xm = clampi(mx - 1, 0, w - 1) - ox_b, xc = mx - ox_b, xp = clampi(mx + 1, 0, w - 1) - ox_b;
            const int sgx = (s_b[ym][xp] + 2 * s_b[yc][xp] + s_b[yp][xp]) - (s_b[ym][xm] + 2 * s_b[yc][xm] + s_b[yp][xm]);
            const int sgy = (s_b[yp][xm] + 2 * s_b[yp][xc] + s_b[yp][xp]) - (s_b[ym][xm] + 2 * s_b[ym][xc] + s_b[ym][xp]);
            m2 = sgx * sgx + sgy * sgy;
        }
        s_m2[ry][rx] = m2;
    }
    __syncthreads();

    // stage 4: non-maximum suppression + class, colour variance
    int cls[kPrepPx];
    unsigned long long local_sum = 0ull;
#pragma unroll
    for (int q = 0; q < kPrepPx; ++q) {
        const int ty = (tid + q * kPrepThreads) / kTile;
        const int gy = y0 + ty;
        cls[q] = 0;
        if (gy < h && gx < w) {
            // gradient at the pixel (recomputed; cheaper than keeping two more LDS planes)
            const int ym = clampi(gy - 1, 0, h - 1) - oy_b, yc = gy - oy_b, yp = clampi(gy + 1, 0, h - 1) - oy_b;
            const int xm = clampi(gx - 1, 0, w - 1) - ox_b, xc = gx - ox_b, xp = clampi(gx + 1, 0, w - 1) - ox_b;
            const int sgx = (s_b[ym][xp] + 2 * s_b[yc][xp] + s_b[yp][xp]) - (s_b[ym][xm] + 2 * s_b[yc][xm] + s_b[yp][xm]);
            const int sgy = (s_b[yp][xm] + 2 * s_b[yp][xc] + s_b[yp][xp]) - (s_b[ym][xm] + 2 * s_b[ym][xc] + s_b[ym][xp]);
            const int m2 = sgx * sgx + sgy * sgy;
            const int ax = abs(sgx), ay = abs(sgy);
            const int s2 = (ax + ay) * (ax + ay);
            int dy1, dx1;                     // first-listed neighbour; the second is its mirror
            if (s2 < 2 * sgx * sgx) { dy1 = 0; dx1 = -1; }
            else if (s2 < 2 * sgy * sgy) { dy1 = -1; dx1 = 0; }
            else if (sgx * sgy > 0) { dy1 = -1; dx1 = -1; }
            else { dy1 = -1; dx1 = 1; }
            const int n1 = s_m2[ty + 1 + dy1][tx + 1 + dx1];
            const int n2 = s_m2[ty + 1 - dy1][tx + 1 - dx1];
            if (m2 > n1 && m2 >= n2) cls[q] = m2 >= hi2 ? 2 : (m2 >= lo2 ? 1 : 0);

            cls_out[(size_t)gy * w + gx] = (uint8_t)cls[q];
        }
        s_cls[ty][tx] = (uint8_t)cls[q];
    }
    // 5x5 colour variance, 25 * sum v^2 - (sum v)^2 per channel, with its own pixel mapping: a thread
    // takes a strip of four pixels of one tile row.  The cells of s_lab already hold the colour at the
    // clamped image coordinate, so the window of pixel (ty, sx + i) is rows ty .. ty + 4, columns
    // sx + i .. sx + i + 4 of the region: two aligned words per row cover all four windows, and
    // sums and sums of squares of four bytes at a time are byte dot products.
    {
        const int vy = tid >> 3, sx = (tid & 7) * 4;
        const int gy = y0 + vy, gx0 = x0 + sx;
        uint32_t v[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            uint32_t s1[4] = {0u, 0u, 0u, 0u}, s2[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int a = 0; a < 5; ++a) {
                const uint32_t* rowp = reinterpret_cast<const uint32_t*>(&s_lab[c][vy + a][sx]);
                const uint32_t w0 = rowp[0], w1 = rowp[1];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t a4 = i == 0 ? w0 : __builtin_amdgcn_alignbyte(w1, w0, i);     // columns i .. i + 3
                    const uint32_t b5 = (w1 >> (8 * i)) & 0xFFu;                                   // column i + 4
                    s1[i] = __builtin_amdgcn_udot4(a4, 0x01010101u, s1[i], false) + b5;
                    s2[i] = __builtin_amdgcn_udot4(a4, a4, s2[i], false) + b5 * b5;
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] += 25u * s2[i] - s1[i] * s1[i];
        }
        if (gy < h) {
            uint32_t* dst = var_out + (size_t)gy * w + gx0;
            if (gx0 + 3 < w && (w & 3) == 0) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(v[0], v[1], v[2], v[3]);
                local_sum += (unsigned long long)v[0] + v[1] + v[2] + v[3];
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (gx0 + i < w) {
                        dst[i] = v[i];
                        local_sum += v[i];
                    }
            }
        }
    }
    // block sum of V -> one atomic
    for (int off = 32; off > 0; off >>= 1) local_sum += __shfl_down(local_sum, off);
    if ((tid & 63) == 0) s_sum[tid >> 6] = local_sum;
    __syncthreads();
    if (tid == 0) {
        unsigned long long t = 0ull;
        for (int k = 0; k < kPrepThreads / 64; ++k) t += s_sum[k];
        atomicAdd(msum_acc, t);
    }

    // hysteresis, tile-local part: union-find in LDS over horizontal runs.
    // A wave holds two tile rows (lanes 0-31 and 32-63), so the run a pixel lies in and the run's
    // smallest key (its leftmost strong pixel, else its leftmost pixel) follow from two ballots.
    uint32_t head_key[kPrepPx];
    bool left_is_cand[kPrepPx];
#pragma unroll
    for (int q = 0; q < kPrepPx; ++q) {
        const int p = tid + q * kPrepThreads;
        const int ty = p / kTile;
        const unsigned long long cand64 = __ballot(cls[q] != 0);
        const unsigned long long strong64 = __ballot(cls[q] == 2);
        const uint32_t row_c = (uint32_t)((tid & 32) ? (cand64 >> 32) : cand64);
        const uint32_t row_s = (uint32_t)((tid & 32) ? (strong64 >> 32) : strong64);
        head_key[q] = (uint32_t)p | (cls[q] == 1 ? kWeakBit : 0u);
        left_is_cand[q] = false;
        if (cls[q] != 0) {
            const uint32_t zeros = ~row_c;
            const uint32_t below = zeros & ((1u << tx) - 1u);
            const uint32_t above = (tx == 31) ? 0u : (zeros & ~((2u << tx) - 1u));
            const int start = below == 0u ? 0 : 32 - __builtin_clz(below);
            const int end = above == 0u ? 31 : __builtin_ctz(above) - 1;
            const uint32_t run = (end == 31 ? 0xFFFFFFFFu : ((2u << end) - 1u)) & ~((1u << start) - 1u);
            const uint32_t strong_in_run = row_s & run;
            head_key[q] = strong_in_run != 0u ? (uint32_t)(ty * kTile + __builtin_ctz(strong_in_run))
                                              : ((uint32_t)(ty * kTile + start) | kWeakBit);
            left_is_cand[q] = tx > 0 && ((row_c >> (tx - 1)) & 1u) != 0u;
        }
        s_lbl[p] = head_key[q];
    }
    __syncthreads();
    // join runs of adjacent rows through their heads (S, SW, SE neighbours)
#pragma unroll
    for (int q = 0; q < kPrepPx; ++q) {
        const int ty = (tid + q * kPrepThreads) / kTile;
        if (cls[q] == 0 || ty + 1 >= kTile) continue;
#pragma unroll
        for (int dx = -1; dx <= 1; ++dx) {
            const int xx = tx + dx;
            if (xx < 0 || xx >= kTile) continue;
            if (s_cls[ty + 1][xx] == 0) continue;
            // The contact of the two runs is made once, by the leftmost pixel pair that touches:
            if (dx <= 0 && left_is_cand[q]) continue;                        // the left neighbour touches (ty+1, xx) too
            if (dx >= 0 && xx >= 1 && s_cls[ty + 1][xx - 1] != 0) continue;  // this pixel touches (ty+1, xx-1) too
            uf_unite<__HIP_MEMORY_SCOPE_WORKGROUP>(s_lbl, head_key[q],
                                                   uf_load<__HIP_MEMORY_SCOPE_WORKGROUP>(s_lbl, (ty + 1) * kTile + xx));
        }
    }
    __syncthreads();
    // each pixel's global link: the global key of its component's smallest key in this tile
    // (itself for pixels that are no edge candidates).  Tile-local row-major order agrees with
    // image row-major order, so "smallest" means the same in both.
#pragma unroll
    for (int q = 0; q < kPrepPx; ++q) {
        const int p = tid + q * kPrepThreads;
        const int ty = p / kTile;
        if (y0 + ty >= h || gx >= w) continue;
        const uint32_t root = (cls[q] != 0) ? uf_find<__HIP_MEMORY_SCOPE_WORKGROUP>(s_lbl, head_key[q])
                                            : ((uint32_t)p);
        const uint32_t rl = root & ~kWeakBit;
        const size_t rg = (size_t)(y0 + (int)(rl / kTile)) * w + (x0 + (int)(rl % kTile));
        parent_out[(size_t)(y0 + ty) * w + gx] = (uint32_t)rg | (root & kWeakBit);
    }
}

// hysteresis, cross-tile part
__global__ __launch_bounds__(256) void k_union(PrepBatch f, int h, int w) {
    if (*f.skip[blockIdx.z] != 0u) return;          // redundant frame, says the pre-pass
    union_strip(f.cls[blockIdx.z], f.parent[blockIdx.z], h, w, blockIdx.x, blockIdx.y);
}

// Gate (Eq. 6), tier assignment and compaction indices of frame `b` of a launch of `n_frames`, by
// one block of 256 threads, after every patch score and patch motion of the frame has been written:
// n_static = #{dP_i < tau_t}, R = n_static / 576, redundant iff R > theta_R; a frame without
// predecessor (no flow) is never redundant.  The last such block of the launch (arrival counter,
// nobody waits) writes the frame-table rows and advances the pool cursors in video order.
__device__ __forceinline__ void pool_tail(TierShared& sh, int* s_cnt, const PoolBatch& f, int b, int n_frames,
                                          float tau_t, float theta_r, const TierLaunch& tl, uint32_t* batch_done) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // gate: n_static = #{dP_i < tau_t}, R = n_static / 576, redundant iff R > theta_R; a frame
    // without predecessor (no flow) is never redundant
    const bool have_flow = f.flow[b] != nullptr;
    // the scores are asked for now, with the patch motions: one memory round trip instead of two on the
    // critical path of the batch (a redundant frame does not use them)
    const TierScores scores = tier_load_scores(f.scores[b]);
    // a tiled frame's patches are those of all its tiles (entries b0 .. b0 + tiles - 1 of the launch): the
    // block of every tile counts them all and so reaches the frame's one decision on its own
    const int tiles = tl.tiles;
    const int b0 = b - b % tiles;
    int n = 0;
    if (have_flow)
        for (int j = 0; j < tiles; ++j) n += count_static(f.dp[b0 + j], tau_t);
    for (int off = 32; off > 0; off >>= 1) n += __shfl_down(n, off);
    if (lane == 0) s_cnt[wave] = n;
    __syncthreads();
    const int n_static = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
    const float r = (float)n_static / (float)(kTokens * tiles);
    const bool redundant = have_flow && r > theta_r;
    TierCounts tc = {};
    tc.state = 1;
    if (!redundant)
        tc = tier_rank(sh, scores, tl.tp, tl.tier + (size_t)b * kTokens, tl.slot + (size_t)b * kTokens,
                       tl.order + (size_t)b * kTokens);
    __syncthreads();
    if (threadIdx.x == 0) {
        sali_gate gt;
        gt.n_static = n_static;
        gt.r_frame = have_flow ? r : 0.0f;
        gt.redundant = redundant ? 1 : 0;
        gt.reserved = 0;
        *f.gate[b] = gt;
        int32_t* out = reinterpret_cast<int32_t*>(f.tcounts[b]);
        __hip_atomic_store(out + 0, tc.state, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int t = 0; t < 4; ++t)
            __hip_atomic_store(out + 1 + t, tc.cnt[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int j = 0; j < 3; ++j)
            __hip_atomic_store(out + 5 + j, tc.q[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();                // counts, tiers, slots and order lists before the arrival
        const bool last = atomicAdd(batch_done, 1u) == (uint32_t)n_frames - 1u;
        if (last) {
            __threadfence();
            *batch_done = 0u;
        }
        s_cnt[0] = last ? 1 : 0;
    }
    __syncthreads();
    if (s_cnt[0] == 0) return;
    if (tl.tp.mode != 2) {
        // every hand-over record by a thread of its own (one round trip), then the rows by one thread with
        // the cursors in registers; the loop is kept rolled: sixteen copies of the commit step are more
        // code than this one wave should have to fetch
        TierCounts* all = reinterpret_cast<TierCounts*>(&sh);
        static_assert(sizeof(TierCounts) * kMaxBatch <= sizeof(TierShared), "records fit the ranking's memory");
        if ((int)threadIdx.x < n_frames) {
            const int32_t* in = reinterpret_cast<const int32_t*>(f.tcounts[threadIdx.x]);
            TierCounts rec = {};
            rec.state = __hip_atomic_load(in + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int t = 0; t < 4; ++t) rec.cnt[t] = __hip_atomic_load(in + 1 + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            all[threadIdx.x] = rec;
        }
        CursorRegs cr = {};
        if (threadIdx.x == 0) cr = cursor_load(tl.cur);
        __syncthreads();
        if (threadIdx.x != 0) return;
#pragma unroll 1
        for (int i = 0; i < n_frames; ++i)
            tier_commit_one(all[i], tl.frame_id + i, tl.rows, cr, tl.cap16, tl.cap8, tl.cap4, tl.cur, tl.budget,
                            tl.tiles);
        cursor_store(tl.cur, cr);
        return;
    }
    // Adaptive thresholds: the ranking above gave each frame's quantiles; its tiers depend on the
    // thresholds the frame before it left, so this block assigns them frame by frame (576 compares and
    // the compaction indices per frame, the whole block) and thread 0 commits and moves the thresholds.
    CursorRegs cr = {};
    if (threadIdx.x == 0) cr = cursor_load(tl.cur);
    if (threadIdx.x < 3) sh.tau[threadIdx.x] = tl.cur->adapt_tau[threadIdx.x];
    __syncthreads();
    for (int i = 0; i < n_frames; ++i) {
        // the frame's hand-over record, the same words for every thread
        const int32_t* in = reinterpret_cast<const int32_t*>(f.tcounts[i]);
        TierCounts tci = {};
        tci.state = __hip_atomic_load(in + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int q[3];
#pragma unroll
        for (int j = 0; j < 3; ++j) q[j] = __hip_atomic_load(in + 5 + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool ranked = tci.state == 3;
        if (ranked)
            tci = tier_assign_adaptive(sh, tier_load_scores(f.scores[i]), tl.tier + (size_t)i * kTokens,
                                       tl.slot + (size_t)i * kTokens, tl.order + (size_t)i * kTokens);
        __syncthreads();
        if (threadIdx.x == 0) {
            const bool stored = tier_commit_one(tci, tl.frame_id + i, tl.rows, cr, tl.cap16, tl.cap8, tl.cap4, tl.cur,
                                                tl.budget, tl.tiles);
            if (ranked && stored) tier_adapt_update(sh, q, tl.tp.adapt_q8);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        cursor_store(tl.cur, cr);
#pragma unroll
        for (int j = 0; j < 3; ++j) tl.cur->adapt_tau[j] = sh.tau[j];
    }
}

// Eq. 5 motion (kMotion) or Eq. 7 score (!kMotion) of each patch.  kWaves = 1: one wave per patch, four
// patches per block of 256 threads (small patches); kWaves = 4: the whole block works on one patch (large
// frames).  The chained step launches the motion variant after the flow and the score variant after the
// saliency pre-pass; a frame that the reuse rule finds redundant gets no scores (Algorithm 1).
// The gate and the tiers (pool_tail) are a further, small launch.  Doing them in the last block of a
// frame to finish (arrival counter) saves that launch but needs a device-scope fence per block, and
// such a fence writes back and invalidates the issuing XCD's L2: with 144 blocks per frame it made the
// K/V kernels running next to it 7 % slower (5 400 -> 5 700 frames/s without), and at 1920x1080 (576
// blocks per frame) it cost the pooling kernel itself 110 us per four-frame launch against 33 us of work.
template <int kWaves, bool kMotion>
__global__ __launch_bounds__(kTierThreads) void k_pool(PoolBatch f, int h, int w, uint8_t* __restrict__ salmap) {
    static_assert(kTierThreads == 256, "four waves, one patch each");
    static_assert(kWaves == 1 || kWaves == 4, "");
    __shared__ uint32_t s_pq[kTierThreads / 64];
    __shared__ float s_pm[kTierThreads / 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (!kMotion && *f.skip[blockIdx.y] != 0u) return;      // redundant frame, says the pre-pass
    {
        // blockIdx.y = frame of the batch
        const uint8_t* __restrict__ cls = f.cls[blockIdx.y];
        const uint32_t* __restrict__ parent = f.parent[blockIdx.y];
        const uint32_t* __restrict__ var = f.var[blockIdx.y];
        const float2* __restrict__ flow = f.flow[blockIdx.y];
        const int token = kWaves == 1 ? blockIdx.x * 4 + wave : blockIdx.x;
        const int pr = token / kGrid, pc = token % kGrid;
        const int ya = (pr * h) / kGrid, yb = ((pr + 1) * h) / kGrid;
        const int xa = (pc * w) / kGrid, xb = ((pc + 1) * w) / kGrid;
        const int pw = xb - xa, area = pw * (yb - ya);
        if (kMotion && flow == nullptr) {           // no predecessor: no motion
            if (lane == 0 && (kWaves == 1 || wave == 0))
                __hip_atomic_store(f.dp_out[blockIdx.y] + token, 0.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        unsigned long long m = 0ull;
        if (!kMotion) m = *f.msum[blockIdx.y];
        const unsigned long long hw = (unsigned long long)h * (unsigned long long)w;
        uint32_t q = 0;
        float mag = 0.0f;
        // four pixels per pass, all their loads issued before any is used (the loop is bound by
        // memory latency, not by work)
        constexpr int kStride = 64 * kWaves, kUnroll = 4;
        for (int p0 = (kWaves == 1 ? lane : (int)threadIdx.x); p0 < area; p0 += kStride * kUnroll) {
            size_t gi[kUnroll];
            int c[kUnroll];
            uint32_t v[kUnroll];
            float2 d[kUnroll];
            bool ok[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int p = p0 + u * kStride;
                ok[u] = p < area;
                const int pp = ok[u] ? p : 0;
                gi[u] = (size_t)(ya + pp / pw) * w + (xa + pp % pw);
                if (kMotion) {
                    d[u] = flow[gi[u]];
                } else {
                    c[u] = cls[gi[u]];
                    v[u] = var[gi[u]];
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                if (!ok[u]) continue;
                if (kMotion) {
                    mag += d[u].x * d[u].x + d[u].y * d[u].y;
                } else {
                    uint32_t e = 0;
                    if (c[u] == 2) e = 1;
                    else if (c[u] == 1) e = (uf_find_settled(parent, (uint32_t)gi[u] | kWeakBit) & kWeakBit) ? 0u : 1u;
                    const uint32_t cm = ((unsigned long long)v[u] * hw > m && v[u] >= kVMin) ? 1u : 0u;
                    q += e + cm;
                    if (salmap != nullptr) salmap[gi[u]] = (uint8_t)(e + cm);
                }
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            if (kMotion) mag += __shfl_down(mag, off);
            else q += __shfl_down(q, off);
        }
        if (kWaves == 4) {
            if (lane == 0) {
                s_pq[wave] = q;
                s_pm[wave] = mag;
            }
            __syncthreads();
            q = s_pq[0] + s_pq[1] + s_pq[2] + s_pq[3];
            mag = (s_pm[0] + s_pm[1]) + (s_pm[2] + s_pm[3]);
        }
        if (lane == 0 && (kWaves == 1 || wave == 0)) {
            if (kMotion) {
                __hip_atomic_store(f.dp_out[blockIdx.y] + token, sqrtf(mag / (float)area), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            } else {
                const uint32_t s_fix = (uint32_t)(((unsigned long long)q << 15) / (unsigned long long)area);
                const float score = (float)s_fix * (1.0f / 65536.0f);      // exact: s_fix <= 2^16
                __hip_atomic_store(f.scores[blockIdx.y] + token, score, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// the tail as a launch of its own: one block per frame
__global__ __launch_bounds__(kTierThreads) void k_pool_tail(PoolBatch f, float tau_t, float theta_r, TierLaunch tl,
                                                            uint32_t* batch_done) {
    __shared__ TierShared sh;
    __shared__ int s_cnt[kTierThreads / 64];
    pool_tail(sh, s_cnt, f, (int)blockIdx.x, (int)gridDim.x, tau_t, theta_r, tl, batch_done);
}

// ---------------------------------------------------------------------------------------------
hipError_t launch_gray(const PrepBatch& f, int n, int h, int w, hipStream_t s) {
    const int px = h * w;
    hipLaunchKernelGGL(k_gray, dim3((px + 4095) / 4096, n), dim3(256), 0, s, f, px);
    return hipGetLastError();
}

hipError_t launch_prep(const PrepBatch& f, int n, int h, int w, GateParams gp, const uint16_t* d_lut,
                       int lo2, int hi2, hipStream_t s) {
    dim3 grid((w + kTile - 1) / kTile, (h + kTile - 1) / kTile, n);
    hipLaunchKernelGGL(k_prep, grid, dim3(kPrepThreads), 0, s, f, h, w, gp,
                       reinterpret_cast<const uint32_t*>(d_lut), lo2, hi2);
    return hipGetLastError();
}

hipError_t launch_union(const PrepBatch& f, int n, int h, int w, hipStream_t s) {
    dim3 grid((w + 63) / 64, (h + 3) / 4, n);
    hipLaunchKernelGGL(k_union, grid, dim3(256), 0, s, f, h, w);
    return hipGetLastError();
}

hipError_t launch_motion(const PoolBatch& f, int n, int h, int w, hipStream_t s) {
    // patches of up to 1024 pixels: one wave each
    if ((long long)h * w <= 1024ll * kTokens) {
        hipLaunchKernelGGL((k_pool<1, true>), dim3(kTokens / 4, n), dim3(kTierThreads), 0, s, f, h, w, nullptr);
    } else {
        hipLaunchKernelGGL((k_pool<4, true>), dim3(kTokens, n), dim3(kTierThreads), 0, s, f, h, w, nullptr);
    }
    return hipGetLastError();
}

hipError_t launch_pool(const PoolBatch& f, int n, int h, int w, uint8_t* d_salmap_or_null,
                       const TierLaunch* tier_or_null, GateParams gp, uint32_t* d_done_counter, hipStream_t s) {
    TierLaunch t = {};
    if (tier_or_null != nullptr) t = *tier_or_null;
    if ((long long)h * w <= 1024ll * kTokens) {
        hipLaunchKernelGGL((k_pool<1, false>), dim3(kTokens / 4, n), dim3(kTierThreads), 0, s, f, h, w, d_salmap_or_null);
    } else {
        hipLaunchKernelGGL((k_pool<4, false>), dim3(kTokens, n), dim3(kTierThreads), 0, s, f, h, w, d_salmap_or_null);
    }
    if (tier_or_null != nullptr) {
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_pool_tail, dim3(n), dim3(kTierThreads), 0, s, f, gp.tau_t, gp.theta_r, t, d_done_counter);
    }
    return hipGetLastError();
}

}  // namespace sali
