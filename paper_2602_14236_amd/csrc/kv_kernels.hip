// Tier assignment, compaction indices, mixed-precision K/V pack and unpack for gfx950.
//
// Spatial Filtering via Saliency-Guided Quantization (Eq. 8), Algorithm 1 ("Store (K_i, V_i)
// with precision Q(s_i)"), Implementation Details (symmetric min-max INT8, asymmetric INT4)
// and Just-In-Time Dequantization.
//
// This file must be compiled with -ffp-contract=off: every quantisation step is one IEEE
// fp32 operation (divide, multiply, subtract, round-half-even); the only fused multiply-adds
// are written out: the one of the INT4 dequantiser and the exact integer packing of INT4 codes.
//
// Data movement: a K/V row (one token in one layer / K|V / head) is 128 halves = 256 B and is
// handled by 16 adjacent lanes, 16 B each, so a wave moves four rows per instruction and a
// 32-value quantisation group sits in one lane quad (reductions are two DPP quad swaps).
// Rows are visited in pool order (all FP16 tokens, then INT8, then INT4, in token order inside
// a tier), so pool writes are contiguous runs and pruned tokens are never read.  A wave covers a
// run of 8 consecutive pool rows (two per lane group, in both kernels) and each of its memory
// instructions four consecutive rows of it (lane group k of the wave takes rows k, k + 4, ...):
// the 64-byte INT4 code rows and the 16- and 8-byte scale / zero-point rows then fill whole cache
// lines per instruction (all-INT4 frames: pack 5.4 -> 5.7 TB/s, unpack 5.6 -> 6.05 TB/s).

#include "sali_internal.h"
#include "tier_body.h"

namespace sali {

namespace {

// unpack: two rows per lane group as well (alone it is 2-6 % faster than with four: 83.8 against
// 86.0 us per frame of the 7B shape, and it leaves more registers to the kernels of other streams)
constexpr int kRowsPerLaneGroup = 2;
constexpr int kRowsPerBlock = 16 * kRowsPerLaneGroup;
// Pack: two rows per lane group, 32 per block.  With four (all other things equal) the kernel is 3 %
// faster when it has the GPU to itself (83 against 86 us per frame of the 7B shape), but it then
// needs 52 registers instead of 34, and next to it the image-analysis kernels of other streams
// (61 to 120 registers) hardly get onto a compute unit while it runs: analysis + store without
// read-back reaches 8 900 frames/s with four rows and 10 750 (69 % of HBM peak) with two; with the
// read-back in the step 5 630 against 5 710.  Three rows (43 registers) behave like four.
constexpr int kPackRows = 2;

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
// max over a quad of values >= 0 (never NaN): their bit patterns order like the numbers
__device__ __forceinline__ float quad_max_nonneg(float v) {
    uint32_t b = __builtin_bit_cast(uint32_t, v);
    b = max(b, (uint32_t)__builtin_amdgcn_mov_dpp((int)b, 0xB1, 0xF, 0xF, true));
    b = max(b, (uint32_t)__builtin_amdgcn_mov_dpp((int)b, 0x4E, 0xF, 0xF, true));
    return __builtin_bit_cast(float, b);
}
// the value held by the odd lane of each lane pair (quad_perm [1, 1, 3, 3])
__device__ __forceinline__ float quad_from_odd(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xF5, 0xF, 0xF, true));
}
// 1.5 * 2^23: adding it to |p| < 2^22 rounds p to the nearest integer (ties to even) and leaves that
// integer, two's complement, in the low mantissa bits of the sum
constexpr float kRoundMagic = 12582912.0f;
// the low bytes of four words, a in bits 0..7 up to d in bits 24..31
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    const uint32_t ab = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);      // bytes: 0 = a.b0, 1 = b.b0, 2 = 3 = zero
    const uint32_t cd = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
    return ab | (cd << 16);
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Tier + rank + compaction indices: one block of 256 threads (see tier_body.h).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kTierThreads) void k_tier(const float* __restrict__ scores, const sali_gate* gate,
                                                  TierParams tp, int frame_id, sali_frame_row* rows,
                                                  uint8_t* __restrict__ tier_out, uint16_t* __restrict__ slot_out,
                                                  uint16_t* __restrict__ order_out, Cursors* cur, int cap16,
                                                  int cap8, int cap4, int budget, int tiles) {
    __shared__ TierShared sh;
    const bool redundant = gate != nullptr && gate->redundant != 0;
    tier_body(sh, scores, redundant, tp, frame_id, rows, tier_out, slot_out, order_out, cur, cap16, cap8, cap4, budget,
              tiles);
}

// ---------------------------------------------------------------------------------------------
// Pack: grid (576 / (16 * kRows), planes, frames); plane = (layer, K|V, head); frame i of the launch has
// id first_frame_id + i.
// ---------------------------------------------------------------------------------------------
// kNTL / kNTS: non-temporal loads / stores
//
// Instruction budget.  The kernel streams at HBM speed only while its vector ALU work stays well
// under the memory time, so the per-row arithmetic is kept short without changing one result bit:
//   * inf/NaN detection is integer work on the packed halves: (w & 0x7FFF7FFF) + 0x04000400 has bit
//     15 (31) set exactly when the low (high) half has an all-ones exponent; the sums of all rows of
//     a thread are OR-ed and tested once;
//   * the two IEEE divisions of a group (scale = m / 127, inv = 127 / m) are shared by a lane pair:
//     even lanes divide for the scale, odd lanes for the inverse, one quad permute hands the
//     inverse over (every lane of a quad holds the same m, so the quotients are the same numbers);
//   * round-half-even of x * inv is the fp32 addition of 1.5 * 2^23, whose low mantissa bits are the
//     two's-complement integer; |x * inv| <= 127 (1 + 2^-22) rounds to at most 127, so the clamp to
//     [-127, 127] of the definition never acts on finite input and is not executed.  INT4 likewise:
//     0 <= (x - min) * inv <= 15 (1 + 2^-22); its eight codes are packed with exact fp32
//     multiply-adds (integers below 2^16) before one conversion.
//   A group that holds an inf or NaN raises SALI_FAULT_NONFINITE; its codes are then unspecified.
template <bool kNTL, bool kNTS, int kRows>
__global__ __launch_bounds__(256) void k_pack(KvBatch f, const sali_frame_row* __restrict__ rows, int first_frame_id,
                                              const uint16_t* __restrict__ order_base, Pools pools, Cursors* cur) {
    const int bz = blockIdx.z;
    const int frame_id = first_frame_id + bz;
    const uint16_t* __restrict__ order = order_base + (size_t)frame_id * kTokens;
    const sali_frame_row row = rows[frame_id];
    if (row.stored == 0) return;
    const int n16 = row.n16, n8 = row.n8;
    const int nkeep = n16 + n8 + row.n4;
    const int j0 = blockIdx.x * (16 * kRows);
    if (j0 >= nkeep) return;
    const size_t plane = blockIdx.y;
    const int g = threadIdx.x >> 4;     // lane group: rows 4 r + (g & 3) of its wave's run
    const int l = threadIdx.x & 15;     // 16-byte chunk of the row
    // the bases of this frame's rows of this plane are uniform (scalar registers); offsets from them fit 32 bits
    const char* __restrict__ kv_plane = reinterpret_cast<const char*>(f.kv[bz]) + plane * (size_t)(kTokens * kHeadDim * 2);
    const size_t r16 = pool_row0(pools, row.base16, n16, plane), r8 = pool_row0(pools, row.base8, n8, plane),
                 r4 = pool_row0(pools, row.base4, row.n4, plane);
    char* __restrict__ p16_plane = reinterpret_cast<char*>(pools.p16) + r16 * (kHeadDim * 2);
    char* __restrict__ c8_plane = reinterpret_cast<char*>(pools.c8) + r8 * kHeadDim;
    char* __restrict__ c4_plane = reinterpret_cast<char*>(pools.c4) + r4 * (kHeadDim / 2);
    float* __restrict__ s8_plane = pools.s8 + r8 * kGroupsPerRow;
    float* __restrict__ s4_plane = pools.s4 + r4 * kGroupsPerRow;
    uint16_t* __restrict__ z4_plane = pools.z4 + r4 * kGroupsPerRow;

    // Three phases, so that the in-order memory counter never makes a wave wait for more than it
    // needs: (1) all row loads are issued back to back (after the token ids of all the
    // lane group's rows have been read from the order table), and rows past the end re-read the
    // block's first row instead of branching; (2) the rows are quantised in registers as their loads
    // arrive, with no memory operation in between; (3) all stores are issued.
    uint32_t tok[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) tok[r] = order[min(j0 + 4 * kRows * (g >> 2) + 4 * r + (g & 3), kTokens - 1)];
    const uint32_t tok_first = order[j0];
    Row16B v[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int j = j0 + 4 * kRows * (g >> 2) + 4 * r + (g & 3);
        const uint32_t off = (j < nkeep ? tok[r] : tok_first) * (kHeadDim * 2) + (uint32_t)l * 16u;
        const u32x4* src = reinterpret_cast<const u32x4*>(kv_plane + off);
        v[r].u = kNTL ? __builtin_nontemporal_load(src) : *src;
    }

    uint32_t expo = 0;                  // bit 15 / 31 set <=> some half of this thread's rows is inf or NaN
    const bool odd = (l & 1) != 0;
    // (a quantised row needs one or two of its four registers for the codes: the group's scale goes to
    // word z, the INT4 zero-point to word y, which keeps the register count down)
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int j = j0 + 4 * kRows * (g >> 2) + 4 * r + (g & 3);
        // rows past the end hold a copy of the block's first row and are quantised like any other (and
        // not stored): a skip here would leave a path on which the row's load is never waited for, and
        // the stores below would then each wait for the whole memory counter
        expo |= (v[r].u.x & 0x7FFF7FFFu) + 0x04000400u;
        expo |= (v[r].u.y & 0x7FFF7FFFu) + 0x04000400u;
        expo |= (v[r].u.z & 0x7FFF7FFFu) + 0x04000400u;
        expo |= (v[r].u.w & 0x7FFF7FFFu) + 0x04000400u;
        if (j < n16) {
            // FP16 tier: verbatim copy
        } else if (j < n16 + n8) {
            // INT8, symmetric: scale = max|x| / 127, q = rne(x * (127 / max|x|))
            float x[8];
            float m = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[e] = (float)v[r].h[e];
                m = fmaxf(m, fabsf(x[e]));
            }
            m = quad_max_nonneg(m);
            const bool nz = m > 0.0f;
            const float quot = (odd ? 127.0f : m) / (odd ? m : 127.0f);      // even lanes: scale, odd lanes: inverse
            const float mine = nz ? quot : 0.0f;
            const float inv = quad_from_odd(mine);
            uint32_t t[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = __builtin_bit_cast(uint32_t, x[e] * inv + kRoundMagic);
            v[r].u.x = pack_low_bytes(t[0], t[1], t[2], t[3]);
            v[r].u.y = pack_low_bytes(t[4], t[5], t[6], t[7]);
            v[r].u.z = __builtin_bit_cast(uint32_t, mine);
        } else {
            // INT4, asymmetric: scale = (max - min) / 15, q = rne((x - min) * (15 / (max - min)))
            float x[8];
            float mn = (float)v[r].h[0], mx = mn;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[e] = (float)v[r].h[e];
                mn = fminf(mn, x[e]);
                mx = fmaxf(mx, x[e]);
            }
            mn = quad_min(mn);
            mx = quad_max(mx);
            const float range = mx - mn;
            const bool nz = range > 0.0f;
            const float quot = (odd ? 15.0f : range) / (odd ? range : 15.0f);
            const float mine = nz ? quot : 0.0f;
            const float inv = quad_from_odd(mine);
            float q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) q[e] = rintf((x[e] - mn) * inv);
            // element 2k low nibble, 2k+1 high nibble of byte k: exact integer arithmetic in fp32
            const float lo = __builtin_fmaf(__builtin_fmaf(__builtin_fmaf(q[3], 16.0f, q[2]), 16.0f, q[1]), 16.0f, q[0]);
            const float hi = __builtin_fmaf(__builtin_fmaf(__builtin_fmaf(q[7], 16.0f, q[6]), 16.0f, q[5]), 16.0f, q[4]);
            v[r].u.x = (uint32_t)lo | ((uint32_t)hi << 16);
            v[r].u.z = __builtin_bit_cast(uint32_t, mine);
            v[r].u.y = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)mn);
        }
    }

#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int j = j0 + 4 * kRows * (g >> 2) + 4 * r + (g & 3);
        if (j >= nkeep) continue;
        if (j < n16) {
            u32x4* dst = reinterpret_cast<u32x4*>(p16_plane + ((uint32_t)j * (kHeadDim * 2) + (uint32_t)l * 16u));
            if (kNTS) __builtin_nontemporal_store(v[r].u, dst); else *dst = v[r].u;
        } else if (j < n16 + n8) {
            const uint32_t prow = (uint32_t)(j - n16);
            u32x2* dst = reinterpret_cast<u32x2*>(c8_plane + (prow * (uint32_t)kHeadDim + (uint32_t)l * 8u));
            const u32x2 codes = {v[r].u.x, v[r].u.y};
            if (kNTS) __builtin_nontemporal_store(codes, dst); else *dst = codes;
            const uint32_t scale_bits = v[r].u.z;       // (a copy: bit_cast of a vector element reads element 0)
            if ((l & 3) == 0) s8_plane[prow * (uint32_t)kGroupsPerRow + (uint32_t)(l >> 2)] = __builtin_bit_cast(float, scale_bits);
        } else {
            const uint32_t prow = (uint32_t)(j - n16 - n8);
            uint32_t* dst = reinterpret_cast<uint32_t*>(c4_plane + (prow * (uint32_t)(kHeadDim / 2) + (uint32_t)l * 4u));
            if (kNTS) __builtin_nontemporal_store(v[r].u.x, dst); else *dst = v[r].u.x;
            const uint32_t scale_bits = v[r].u.z;
            if ((l & 3) == 0) {
                s4_plane[prow * (uint32_t)kGroupsPerRow + (uint32_t)(l >> 2)] = __builtin_bit_cast(float, scale_bits);
                z4_plane[prow * (uint32_t)kGroupsPerRow + (uint32_t)(l >> 2)] = (uint16_t)v[r].u.y;
            }
        }
    }
    if ((expo & 0x80008000u) != 0) atomicOr(&cur->status, SALI_FAULT_NONFINITE);
}

// ---------------------------------------------------------------------------------------------
// Dequantise-on-read of the pool rows of one lane group.  kTier >= 0: every row of
// the wave is of that tier (0 FP16, 1 INT8, 2 INT4, 3 pruned); kTier < 0: tiers are tested per row.
// Three phases as in the pack kernel: all loads, then the arithmetic, then the stores.
struct UnpackPlanes {
    const char* p16;
    const char* c8;
    const char* c4;
    const float* s8;
    const float* s4;
    const uint16_t* z4;
    char* out;
};

template <bool kNTL, bool kNTS, int kTier>
__device__ __forceinline__ void unpack_rows(const UnpackPlanes& pl, const sali_frame_row& row,
                                            const uint16_t* __restrict__ order, uint8_t* valid, bool first_plane,
                                            int j0, int g, int l) {
    const int n16 = row.n16, n8 = row.n8, n4 = row.n4;
    uint32_t tok[kRowsPerLaneGroup];
#pragma unroll
    for (int r = 0; r < kRowsPerLaneGroup; ++r) tok[r] = order[j0 + 4 * kRowsPerLaneGroup * (g >> 2) + 4 * r + (g & 3)];
    Row16B raw[kRowsPerLaneGroup];
    float scale[kRowsPerLaneGroup];
    uint16_t zbits[kRowsPerLaneGroup];
    int tier[kRowsPerLaneGroup];
#pragma unroll
    for (int r = 0; r < kRowsPerLaneGroup; ++r) {
        const int j = j0 + 4 * kRowsPerLaneGroup * (g >> 2) + 4 * r + (g & 3);          // always < 576
        tier[r] = kTier >= 0 ? kTier : (j < n16 ? 0 : (j < n16 + n8 ? 1 : (j < n16 + n8 + n4 ? 2 : 3)));
        raw[r].u = zero4();
        scale[r] = 0.0f;
        zbits[r] = 0;
        if (tier[r] == 0) {
            const u32x4* srcp = reinterpret_cast<const u32x4*>(pl.p16 + ((uint32_t)j * (kHeadDim * 2) + (uint32_t)l * 16u));
            raw[r].u = kNTL ? __builtin_nontemporal_load(srcp) : *srcp;
        } else if (tier[r] == 1) {
            const uint32_t prow = (uint32_t)(j - n16);
            const u32x2* srcp = reinterpret_cast<const u32x2*>(pl.c8 + (prow * (uint32_t)kHeadDim + (uint32_t)l * 8u));
            const u32x2 c = kNTL ? __builtin_nontemporal_load(srcp) : *srcp;
            raw[r].u.x = c.x;
            raw[r].u.y = c.y;
            scale[r] = pl.s8[prow * (uint32_t)kGroupsPerRow + (uint32_t)(l >> 2)];
        } else if (tier[r] == 2) {
            const uint32_t prow = (uint32_t)(j - n16 - n8);
            const uint32_t* srcp = reinterpret_cast<const uint32_t*>(pl.c4 + (prow * (uint32_t)(kHeadDim / 2) + (uint32_t)l * 4u));
            raw[r].u.x = kNTL ? __builtin_nontemporal_load(srcp) : *srcp;
            scale[r] = pl.s4[prow * (uint32_t)kGroupsPerRow + (uint32_t)(l >> 2)];
            zbits[r] = pl.z4[prow * (uint32_t)kGroupsPerRow + (uint32_t)(l >> 2)];
        }
    }
#pragma unroll
    for (int r = 0; r < kRowsPerLaneGroup; ++r) {
        Row16B o;
        o.u = raw[r].u;                                         // FP16 tier: as stored; pruned: zeros
        if (tier[r] == 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t word = e < 4 ? raw[r].u.x : raw[r].u.y;
                const int q = (int)(int8_t)((word >> (8 * (e & 3))) & 0xFF);
                o.h[e] = to_half_after_f32((float)q * scale[r]);          // one fp32 multiply, then RNE to fp16
            }
        } else if (tier[r] == 2) {
            const float zero = (float)__builtin_bit_cast(_Float16, zbits[r]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int q = (int)((raw[r].u.x >> (4 * e)) & 0xF);
                o.h[e] = to_half_after_f32(__builtin_fmaf((float)q, scale[r], zero));   // fused: one fp32 rounding
            }
        }
        raw[r].u = o.u;
    }
#pragma unroll
    for (int r = 0; r < kRowsPerLaneGroup; ++r) {
        u32x4* dst = reinterpret_cast<u32x4*>(pl.out + (tok[r] * (uint32_t)(kHeadDim * 2) + (uint32_t)l * 16u));
        if (kNTS) __builtin_nontemporal_store(raw[r].u, dst); else *dst = raw[r].u;
        if (valid != nullptr && first_plane && l == 0) valid[tok[r]] = tier[r] != 3 ? 1 : 0;
    }
}

// ---------------------------------------------------------------------------------------------
// Unpack: grid (576 / kRowsPerBlock, planes, frames); rebuilds the dense fp16 frames in token order; frame i of
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
            const int tok = j0 + 4 * kRowsPerLaneGroup * (g >> 2) + 4 * r + (g & 3);
            out[(plane * kTokens + tok) * 16 + l] = zero4();
            if (valid != nullptr && plane == 0 && l == 0) valid[tok] = 0;
        }
        if (blockIdx.x == 0 && plane == 0 && threadIdx.x == 0) atomicOr(&cur->status, SALI_FAULT_NO_DATA);
        return;
    }
    const sali_frame_row row = rows[src];
    const uint16_t* order = order_base + (size_t)src * kTokens;
    const int n16 = row.n16, n8 = row.n8, n4 = row.n4;
    // the bases of the source frame's rows of this plane are uniform; offsets from them fit 32 bits
    const size_t r16 = pool_row0(pools, row.base16, n16, plane), r8 = pool_row0(pools, row.base8, n8, plane),
                 r4 = pool_row0(pools, row.base4, n4, plane);
    const char* __restrict__ p16_plane = reinterpret_cast<const char*>(pools.p16) + r16 * (kHeadDim * 2);
    const char* __restrict__ c8_plane = reinterpret_cast<const char*>(pools.c8) + r8 * kHeadDim;
    const char* __restrict__ c4_plane = reinterpret_cast<const char*>(pools.c4) + r4 * (kHeadDim / 2);
    const float* __restrict__ s8_plane = pools.s8 + r8 * kGroupsPerRow;
    const float* __restrict__ s4_plane = pools.s4 + r4 * kGroupsPerRow;
    const uint16_t* __restrict__ z4_plane = pools.z4 + r4 * kGroupsPerRow;
    char* __restrict__ out_plane = reinterpret_cast<char*>(out) + plane * (size_t)(kTokens * kHeadDim * 2);

    UnpackPlanes pl = {p16_plane, c8_plane, c4_plane, s8_plane, s4_plane, z4_plane, out_plane};
    // A wave covers 8 consecutive pool rows, nearly always of one tier: those waves take a path
    // without tier branches (the scalar test below), where the compiler can issue all loads back to
    // back and wait for each exactly when it is used; a wave that straddles a tier boundary takes
    // the general path.
    const int w0 = j0 + 4 * kRowsPerLaneGroup * __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int w1 = w0 + 4 * kRowsPerLaneGroup;
    const int e16 = n16, e8 = n16 + n8, e4 = n16 + n8 + n4;
    if (w1 <= e16) unpack_rows<kNTL, kNTS, 0>(pl, row, order, valid, plane == 0, j0, g, l);
    else if (w0 >= e16 && w1 <= e8) unpack_rows<kNTL, kNTS, 1>(pl, row, order, valid, plane == 0, j0, g, l);
    else if (w0 >= e8 && w1 <= e4) unpack_rows<kNTL, kNTS, 2>(pl, row, order, valid, plane == 0, j0, g, l);
    else if (w0 >= e4) unpack_rows<kNTL, kNTS, 3>(pl, row, order, valid, plane == 0, j0, g, l);
    else unpack_rows<kNTL, kNTS, -1>(pl, row, order, valid, plane == 0, j0, g, l);
}

// ---------------------------------------------------------------------------------------------
hipError_t launch_tier(const float* d_scores, const sali_gate* d_gate_or_null, TierParams tp, int frame_id,
                       sali_frame_row* d_rows, uint8_t* d_tier, uint16_t* d_slot, uint16_t* d_order,
                       Cursors* d_cur, Pools pools, int budget, int tiles, hipStream_t s) {
    hipLaunchKernelGGL(k_tier, dim3(1), dim3(kTierThreads), 0, s, d_scores, d_gate_or_null, tp, frame_id, d_rows,
                       d_tier, d_slot, d_order, d_cur, pools.cap16, pools.cap8, pools.cap4, budget, tiles);
    return hipGetLastError();
}

hipError_t launch_pack(const KvBatch& f, int n, const sali_frame_row* d_rows, int first_frame_id,
                       const uint16_t* d_order_base, Pools pools, Cursors* d_cur, int n_planes, hipStream_t s) {
    // streaming both ways: non-temporal loads and stores.  (Ordinary stores keep the new pool rows in
    // the last-level cache, which speeds up an immediate read-back by about as much as it slows this
    // kernel; without an immediate read-back non-temporal stores measured 10 % faster.)
    hipLaunchKernelGGL((k_pack<true, true, kPackRows>), dim3(kTokens / (16 * kPackRows), n_planes, n), dim3(256), 0, s, f,
                       d_rows, first_frame_id, d_order_base, pools, d_cur);
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
