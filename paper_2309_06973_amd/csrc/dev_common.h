// Device helpers shared by the kernels (wave64, gfx950).
#pragma once

#include "internal.h"

namespace shifter {

// Largest t with prefix[t] <= tile; requires prefix[0] <= tile < prefix[n].
// `tile` is uniform over the block, so the search runs on scalar registers.
__device__ __forceinline__ uint32_t find_tensor(const uint32_t* __restrict__ prefix,
                                                uint32_t n, uint32_t tile) {
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (prefix[mid] <= tile) lo = mid; else hi = mid;
    }
    return lo;
}

// Bins of the sample histogram of the single-pass selections: SAMPLE_BINS bins of 2^15 keys
// (1/256 of a binade, 0.27 % of a magnitude) over the 64 binades from 2^-50 to 2^14, where
// the weights of networks live; the keys below that window (zeros among them) share bin 0,
// the keys above it the last bin.  The intervals predicted from the sample are rounded
// outward to whole bins, so narrow bins mean few candidates; no result depends on the
// binning (weights all outside the window only send the selection to its multi-pass form).
constexpr uint32_t SAMPLE_BINS = 16384;
constexpr uint32_t SAMPLE_BIN_SHIFT = 15;
constexpr uint32_t SAMPLE_KEY0 = (127u - 50u) << 23;      // first key of the window
static_assert(((uint64_t)SAMPLE_BINS << SAMPLE_BIN_SHIFT) == (64ull << 23), "64 binades");
__device__ __forceinline__ uint32_t sample_bin(uint32_t key) {
    return key < SAMPLE_KEY0 ? 0u : min((key - SAMPLE_KEY0) >> SAMPLE_BIN_SHIFT, SAMPLE_BINS - 1u);
}
__device__ __forceinline__ uint32_t sample_bin_first_key(uint32_t bin) {
    return bin == 0u ? 0u : SAMPLE_KEY0 + (bin << SAMPLE_BIN_SHIFT);
}
__device__ __forceinline__ uint32_t sample_bin_last_key(uint32_t bin) {
    return bin >= SAMPLE_BINS - 1u ? 0x7fffffffu : SAMPLE_KEY0 + ((bin + 1u) << SAMPLE_BIN_SHIFT) - 1u;
}

// A value that is the same in every lane, moved to scalar registers.  The builtin returns
// a signed int: without the casts the low word of a 64-bit value would be sign-extended.
__device__ __forceinline__ uint32_t uniform_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)x);
}
__device__ __forceinline__ uint64_t uniform_u64(uint64_t x) {
    return ((uint64_t)uniform_u32((uint32_t)(x >> 32)) << 32) | (uint64_t)uniform_u32((uint32_t)x);
}

// Small-quotient division used to index tile-relative flag slots.  The host sets
// magic = floor(2^32 / d) + 1 when 1 < d <= 2 * TILE (exact while x * d < 2^32, and here
// x < d + TILE + 2); for larger d the callers guarantee x < 2 * d.
__device__ __forceinline__ uint32_t div_small(uint32_t x, uint32_t d, uint32_t magic) {
    return d == 1 ? x : (magic ? __umulhi(x, magic) : (x >= d ? 1u : 0u));
}
__device__ __forceinline__ uint32_t mod_small(uint32_t x, uint32_t d, uint32_t magic) {
    return d == 1 ? 0u : (magic ? x - __umulhi(x, magic) * d : (x >= d ? x - d : x));
}

// 16-byte and 4-byte global accesses with an optional non-temporal (streaming) hint:
// arenas larger than the last-level cache are read once and written once per pass, and
// the hint gains about 8 % of copy bandwidth on this chip.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ uint4 load_u4(const uint4* p) {
    const u32x4* q = reinterpret_cast<const u32x4*>(p);
    const u32x4 v = NT ? __builtin_nontemporal_load(q) : *q;
    return make_uint4(v.x, v.y, v.z, v.w);
}
template <bool NT>
__device__ __forceinline__ void store_u4(uint4* p, uint4 v) {
    u32x4 x;
    x.x = v.x; x.y = v.y; x.z = v.z; x.w = v.w;
    u32x4* q = reinterpret_cast<u32x4*>(p);
    if (NT) __builtin_nontemporal_store(x, q); else *q = x;
}
template <bool NT>
__device__ __forceinline__ void store_u1(uint32_t* p, uint32_t v) {
    if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}

__device__ __forceinline__ uint32_t key_of(float w) {
    return __float_as_uint(w) & 0x7fffffffu;
}

// Exclusive scan of one u64 per thread over a block of THREADS threads.
// smem: at least THREADS / 64 + 1 entries.  Contains two barriers.
template <uint32_t THREADS = BLOCK>
__device__ __forceinline__ uint64_t block_excl_scan_u64(uint64_t v, uint64_t* smem,
                                                        uint64_t* total) {
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    unsigned long long x = v;
    for (uint32_t d = 1; d < 64; d <<= 1) {
        const unsigned long long y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    __syncthreads();   // protects smem against a previous use
    if (lane == 63) smem[wid] = x;
    __syncthreads();
    uint64_t woff = 0, tot = 0;
    for (uint32_t i = 0; i < THREADS / 64; ++i) {
        const uint64_t s = smem[i];
        if (i < wid) woff += s;
        tot += s;
    }
    *total = tot;
    return woff + x - v;
}

}  // namespace shifter
