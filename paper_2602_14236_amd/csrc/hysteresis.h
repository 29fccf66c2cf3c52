// Hysteresis of the Canny stage as a lock-free union-find, shared by the saliency kernels
// (Implementation Details: Canny edge detection).
// A pixel's key is its index with bit 31 set for weak pixels; links always point to the smaller
// key, so the root of a component is a strong pixel iff the component has one.
#pragma once

#include "sali_internal.h"

namespace sali {

constexpr int kTile = 32;                       // tile side of the saliency pre-pass
constexpr uint32_t kWeakBit = 0x80000000u;

// union-find on a parent array (LDS or global); key = index | weak bit; links go to smaller keys
template <int kScope>
__device__ __forceinline__ uint32_t uf_load(const uint32_t* parent, uint32_t idx) {
    return __hip_atomic_load(parent + idx, __ATOMIC_RELAXED, kScope);
}

template <int kScope>
__device__ __forceinline__ uint32_t uf_find(const uint32_t* parent, uint32_t key) {
    uint32_t k = key;               // keys strictly decrease along links, so this terminates
    for (;;) {
        const uint32_t p = uf_load<kScope>(parent, k & ~kWeakBit);
        if (p == k) return k;
        k = p;
    }
}

// for kernels that run after all links are final: ordinary cached loads
__device__ __forceinline__ uint32_t uf_find_settled(const uint32_t* __restrict__ parent, uint32_t key) {
    uint32_t k = key;
    for (;;) {
        const uint32_t p = parent[k & ~kWeakBit];
        if (p == k) return k;
        k = p;
    }
}

template <int kScope>
__device__ __forceinline__ void uf_unite(uint32_t* parent, uint32_t ka, uint32_t kb) {
    for (;;) {
        ka = uf_find<kScope>(parent, ka);
        kb = uf_find<kScope>(parent, kb);
        if (ka == kb) return;
        if (ka < kb) { const uint32_t t = ka; ka = kb; kb = t; }      // ka is the larger key
        const uint32_t old = atomicMin(parent + (ka & ~kWeakBit), kb);
        if (old == ka) return;      // ka was a root and now points at kb
        ka = old;                   // somebody linked ka first: continue from where it pointed
    }
}

// Cross-tile part: a strip of 64 x 4 pixels per block of 256 threads; only pixels on a tile border
// have neighbours in another tile of the pre-pass (pairs inside a tile were joined in LDS there).
__device__ __forceinline__ void union_strip(const uint8_t* __restrict__ cls, uint32_t* parent, int h, int w,
                                            int strip_x, int strip_y) {
    const int x = strip_x * 64 + (int)(threadIdx.x & 63);
    const int y = strip_y * 4 + (int)(threadIdx.x >> 6);
    if (x >= w || y >= h) return;
    const int lx = x % kTile, ly = y % kTile;
    if (lx != 0 && lx != kTile - 1 && ly != kTile - 1) return;      // all forward neighbours in the same tile
    const size_t gi = (size_t)y * w + x;
    const int c = cls[gi];
    if (c == 0) return;
    const uint32_t me = (uint32_t)gi | (c == 1 ? kWeakBit : 0u);
    const int ny[4] = {0, 1, 1, 1};
    const int nx[4] = {1, -1, 0, 1};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int yy = y + ny[k], xx = x + nx[k];
        if (yy >= h || xx < 0 || xx >= w) continue;
        if (yy / kTile == y / kTile && xx / kTile == x / kTile) continue;     // joined in LDS already
        const size_t gj = (size_t)yy * w + xx;
        const int cj = cls[gj];
        if (cj == 0) continue;
        uf_unite<__HIP_MEMORY_SCOPE_AGENT>(parent, me, (uint32_t)gj | (cj == 1 ? kWeakBit : 0u));
    }
}

}  // namespace sali
