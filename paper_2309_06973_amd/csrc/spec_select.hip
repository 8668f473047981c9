// Single-pass exact selection of the P-th smallest (|w|, g) pair for one prune count:
// the unstructured magnitude ranking of Sec. II-A / Sec. III-C of the paper, reached in
// one read of the arena instead of one read per radix digit.
//
//   1. sample      a systematic sample of the prunable weights (two 128-byte lines out
//                  of every sampled tile) is histogrammed on the top 16 key bits;
//   2. predict     from the sample's order statistics around P/N, widened by a margin,
//                  a key interval [lo, hi] that should contain the threshold key;
//   3. one pass    over the arena counts the weights below lo and appends the
//                  (key, g) pairs inside [lo, hi] to a candidate buffer.  In the fused
//                  form the same pass already writes the sparse weights, the mask and
//                  the alive flags for every weight outside the interval;
//   4. finish      if  n_below < P <= n_below + n_candidates  the P-th pair is the
//                  (P - n_below)-th candidate: a 256-bin histogram over the candidates,
//                  a 4096-bin one over the selected bin, and an exact rank inside the
//                  last bin give the record; the fused form then settles the candidates.
//
// The result is exact whenever step 4's check holds; otherwise (a sample that misled,
// an interval with too many ties, a full buffer) a status bit is raised and the host
// runs the multi-pass radix select instead.
#include <algorithm>

#include "dev_common.h"

namespace shifter {

constexpr uint32_t SBINS = SAMPLE_BINS;  // sample histogram bins (sample_bin)
constexpr uint32_t FBINS1 = 256;        // round-1 finishing histogram: one bin per thread
constexpr uint32_t FBINS = 4096;        // round-2 finishing histogram (one block, LDS)
constexpr uint32_t FIN_BLOCKS = SPEC_FIN_BLOCKS;  // blocks of the passes over candidates

// Global atomics to one address serialise (about 11 ns each on this chip), so every
// counter that all blocks touch is split into SPEC_SUB copies, one 128-byte line each,
// chosen by blockIdx; the candidate buffer is split the same way.
enum { CNT_CAND = 0, CNT_BELOW = 1 };
__device__ __forceinline__ uint32_t* sub_counter(uint32_t* cnt, uint32_t which, uint32_t sb) {
    return cnt + (which * SPEC_SUB + sb) * 32u;
}

// The sample: from every quarter (1024 weights) of every sample_tile_stride-th tile one
// 64-byte sector of 16 weights, at a position that rotates with the tile and the quarter.
// Every filter of 1024 or more weights is thus sampled in proportion to its size - the
// sample is stratified by filter, which matters because filters differ in scale by
// orders of magnitude and a sample clustered on few filters misjudges the quantiles.
// A wavefront takes four tiles per step (16 lanes per tile, 4 lanes per sector, one
// float4 each).  The samples go to a per-block LDS histogram first: a global atomic
// costs about 11 ns per lane on one address, and the bins around the mode are hot.
__host__ __device__ __forceinline__ uint32_t sample_sector(uint32_t tile, uint32_t quarter) {
    return (tile * 37u + quarter * 11u) & 63u;
}

constexpr uint32_t SAMPLE_THREADS = 1024;   // sixteen wavefronts on the block's CU keep its loads in flight

__global__ __launch_bounds__(SAMPLE_THREADS) void spec_sample_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    const uint16_t* __restrict__ tile_tensor, uint32_t n_tiles, uint32_t tile_stride,
    const float* __restrict__ w, uint32_t* shist, SampleZero z) {
    __shared__ uint32_t h[SBINS];
    if (z.cnt) {
        // scratch of the K-rank ranking, idle until its pass: rows 0 .. k and
        // MAXK + 1 .. MAXK + k of the split counters (the first word of each 128-byte line)
        const uint32_t tid = blockIdx.x * SAMPLE_THREADS + threadIdx.x, nthr = gridDim.x * SAMPLE_THREADS;
        for (uint32_t i = tid; i < (2u * z.k + 1u) * SPEC_SUB; i += nthr) {
            const uint32_t row = i / SPEC_SUB, sb = i % SPEC_SUB;
            const uint32_t r = row <= z.k ? row : MAXK + 1u + (row - (z.k + 1u));
            z.cnt[((size_t)r * SPEC_SUB + sb) * 32u] = 0;
        }
        for (uint32_t i = tid; i < z.k * 256u; i += nthr) z.ghist[i] = 0;
        for (uint32_t i = tid; i < z.extra_n; i += nthr) z.extra[i] = 0;
        if (tid < MAXK) {
            z.list_cnt[tid] = 0;
            z.rout[tid].fail = 0;
        }
    }
    if (z.ss) {
        // set-up of the one-count selection, idle until the kernels behind this one: its
        // split counters and the caller's flag arrays cleared, its state initialised (every
        // ranking leaves the sample histogram cleared, see the predict kernels)
        const uint64_t tid = (uint64_t)blockIdx.x * SAMPLE_THREADS + threadIdx.x;
        const uint64_t stride = (uint64_t)gridDim.x * SAMPLE_THREADS;
        for (uint64_t i = tid; i < 2u * SPEC_SUB * 32u; i += stride) z.cnt1[i] = 0;
        for (uint64_t i = tid; i < z.na; i += stride) z.fa[i] = 0;
        for (uint64_t i = tid; i < z.nb; i += stride) z.fb[i] = 0;
        if (tid == 0) {
            SpecState* ss = z.ss;
            ss->p = z.p;
            ss->n_below = 0;
            ss->n_inside = 0;
            ss->m_valid = z.m_valid;
            ss->status = 0;
            ss->list_cnt = 0;
            ss->lo = 0;
            ss->hi = 0x7fffffffu;
            ss->mid = 0;
            ss->sh = 19;
        }
    }
    for (uint32_t i = threadIdx.x; i < SBINS; i += SAMPLE_THREADS) h[i] = 0;
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = blockIdx.x * (SAMPLE_THREADS / 64) + (threadIdx.x >> 6);
    const uint32_t n_waves = gridDim.x * (SAMPLE_THREADS / 64);
    const uint32_t quarter = (lane >> 2) & 3u, part = lane & 3u;
    // address of this lane's four samples of sampled tile s, or nullptr; the tensor of a
    // tile comes from a table (one load instead of a search per lane)
    auto locate = [&](uint64_t s) -> const float* {
        if (s * tile_stride >= n_tiles) return nullptr;
        const uint32_t tile = (uint32_t)(s * tile_stride);
        const uint32_t t = tile_tensor[tile];
        if (!tens[t].prunable) return nullptr;
        const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
        const uint32_t n = min(TILE, tens[t].numel - e0);
        const uint32_t j = quarter * 1024u + sample_sector(tile, quarter) * 16u + part * 4u;
        return j + 3 < n ? w + tens[t].offset + e0 + j : nullptr;
    };
    auto fetch = [&](const float* p) -> float4 {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p) {
            if ((reinterpret_cast<uintptr_t>(p) & 15u) == 0) {
                x = *reinterpret_cast<const float4*>(p);
            } else {
                x.x = p[0]; x.y = p[1]; x.z = p[2]; x.w = p[3];
            }
        }
        return x;
    };
    auto count = [&](const float* p, const float4& x) {
        if (!p) return;
        atomicAdd(&h[sample_bin(key_of(x.x))], 1u);
        atomicAdd(&h[sample_bin(key_of(x.y))], 1u);
        atomicAdd(&h[sample_bin(key_of(x.z))], 1u);
        atomicAdd(&h[sample_bin(key_of(x.w))], 1u);
    };
    // two sampled tiles per lane group and step, their loads in flight together
    const uint64_t step = (uint64_t)n_waves * 4;
    for (uint64_t s = (uint64_t)wave * 4 + (lane >> 4); s * tile_stride < n_tiles; s += 2 * step) {
        const float* pa = locate(s);
        const float* pb = locate(s + step);
        const float4 xa = fetch(pa);
        const float4 xb = fetch(pb);
        count(pa, xa);
        count(pb, xb);
    }
    __syncthreads();
    // the blocks start at different segments of the histogram: the populated bins are few
    // and neighbours, and atomics that meet at one address take their turns
    constexpr uint32_t SEGS = SBINS / SAMPLE_THREADS;
    for (uint32_t it = 0; it < SEGS; ++it) {
        const uint32_t i = ((it + blockIdx.x) % SEGS) * SAMPLE_THREADS + threadIdx.x;
        const uint32_t c = h[i];
        if (c) atomicAdd(&shist[i], c);
    }
}

// One block: the sample's order statistics around P/N give the candidate interval
// [lo, hi] and a provisional threshold mid (the fused pass writes candidates below mid as
// removed, the others as kept; few of them then need correcting).
// The histogram is read as 64 segments of 256 bins, one coalesced load per wavefront.
__global__ __launch_bounds__(BLOCK) void spec_predict_kernel(SpecState* ss, uint32_t* shist,
                                                             uint64_t n_prunable,
                                                             double margin_sigmas) {
    constexpr uint32_t SEG = 256, NSEG = SBINS / SEG;   // 64 segments
    static_assert(NSEG == 64, "one segment per lane, one segment sum per thread");
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t seg_sum[NSEG];
    __shared__ uint64_t s_base[NSEG];
    __shared__ uint32_t s_bin[3];
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    for (uint32_t sg = wid; sg < NSEG; sg += BLOCK / 64) {
        const uint4 x = reinterpret_cast<const uint4*>(shist + sg * SEG)[lane];
        uint32_t v = x.x + x.y + x.z + x.w;
        for (uint32_t d = 32; d > 0; d >>= 1) v += __shfl_down(v, d, 64);
        if (lane == 0) seg_sum[sg] = v;
    }
    if (threadIdx.x < 3) s_bin[threadIdx.x] = 0xffffffffu;
    __syncthreads();
    const uint64_t mine = threadIdx.x < NSEG ? seg_sum[threadIdx.x] : 0;
    uint64_t total;
    const uint64_t base = block_excl_scan_u64(mine, smem, &total);
    const uint64_t p = ss->p;
    const uint32_t m = ss->m_valid;
    const bool use = p > 0 && m >= 256 && n_prunable > 0 && total == m;
    double r[3] = {0, 0, 0};   // 0-based sample ranks: low end, high end, centre
    if (use) {
        const double frac = (double)p / (double)n_prunable;
        const double centre = frac * (double)m;
        // a multiple of the binomial deviation of a simple random sample of this size
        const double delta = margin_sigmas * sqrt((double)m * frac * (1.0 - frac)) + 16.0;
        r[0] = centre - delta;
        r[1] = centre + delta;
        r[2] = centre;
    }
    // bin holding the r-th sample, one wavefront per rank: the segment from the segment
    // bases (one per lane), then a scan over the segment's 256 bins (four per lane)
    if (threadIdx.x < NSEG) s_base[threadIdx.x] = base;
    __syncthreads();
    if (wid < 3 && use && r[wid] >= 0.0 && r[wid] < (double)m) {
        const uint64_t target = (uint64_t)r[wid];
        const uint32_t sg = (uint32_t)__popcll(__ballot(s_base[lane] <= target)) - 1u;   // bases ascend from 0
        const uint4 x = reinterpret_cast<const uint4*>(shist + sg * SEG)[lane];
        const uint32_t mine4 = x.x + x.y + x.z + x.w;
        uint32_t incl = mine4;
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(incl, d, 64);
            if (lane >= d) incl += y;
        }
        const uint64_t seg_base = s_base[sg];
        const unsigned long long over = __ballot(seg_base + incl > target);
        if (over != 0 && lane == (uint32_t)__ffsll(over) - 1u) {
            uint64_t run = seg_base + incl - mine4;
            const uint32_t v[4] = {x.x, x.y, x.z, x.w};
            for (uint32_t i = 0; i < 4; ++i) {
                run += v[i];
                if (run > target) { s_bin[wid] = sg * SEG + lane * 4 + i; break; }
            }
        }
    }
    __syncthreads();
    // the sample has been read: cleared for the next ranking, which adds to it
    for (uint32_t i = threadIdx.x; i < SBINS; i += BLOCK) shist[i] = 0;
    if (threadIdx.x != 0) return;
    uint32_t lo = 0, hi = 0x7fffffffu;
    if (s_bin[0] != 0xffffffffu) lo = sample_bin_first_key(s_bin[0]);
    if (s_bin[1] != 0xffffffffu && r[1] < (double)(m - 1)) hi = sample_bin_last_key(s_bin[1]);
    uint32_t mid = lo;
    if (s_bin[2] != 0xffffffffu)      // the middle of the bin
        mid = sample_bin_first_key(s_bin[2]) + (sample_bin_last_key(s_bin[2]) - sample_bin_first_key(s_bin[2])) / 2u;
    mid = max(lo, min(mid, hi));
    uint32_t sh = 0;
    while (((hi - lo) >> sh) >= FBINS1) ++sh;
    ss->lo = lo;
    ss->hi = hi;
    ss->mid = mid;
    ss->sh = sh;
}

// The one pass over the arena.  FUSED also writes the sparse weights and the mask of
// every weight (those of the candidates provisionally: removed below mid, kept from mid
// on) and the alive flags of the kept weights outside the candidate interval;
// spec_fixup_kernel settles the candidates.  A candidate pair holds the weight's full bit
// pattern (sign included, so a wrongly removed weight can be restored) and its index.
template <bool FUSED, bool NT>
__global__ __launch_bounds__(BLOCK) void spec_pass_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    uint32_t n_t, const float* __restrict__ w, SpecState* ss, uint32_t* cnt,
    uint2* __restrict__ cand, uint32_t cap_sb, float* __restrict__ w_out,
    uint8_t* __restrict__ mask, uint8_t* out_alive, uint8_t* in_alive) {
    __shared__ uint8_t rowf[FUSED ? TILE + 16 : 16];
    __shared__ uint8_t colf[FUSED ? TILE + 16 : 16];
    __shared__ uint32_t s_below, s_nan, s_base, s_wtot[BLOCK / 64];

    const uint32_t tile = blockIdx.x;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    const DevTensor T = tens[t];
    if (!FUSED && !T.prunable) return;
    const bool ranked = T.prunable != 0 && ss->p != 0;   // P = 0: nothing is removed
    const uint32_t lo = ss->lo, hi = ss->hi, mid = ss->mid;
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const uint32_t g0 = (uint32_t)(T.gbase + e0);
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    const uint32_t sb = blockIdx.x & (SPEC_SUB - 1);
    uint2* my_cand = cand + (size_t)sb * cap_sb;
    uint32_t c0 = 0, r0 = 0, nrows = 0, ncols = 0;
    if (threadIdx.x == 0) { s_below = 0; s_nan = 0; s_base = 0; }
    if (FUSED) {
        c0 = e0 % T.khw;
        r0 = e0 % T.row_len;
        nrows = (r0 + n - 1) / T.row_len + 1;
        ncols = (c0 + n - 1) / T.khw + 1;
        for (uint32_t s = threadIdx.x; s < nrows; s += BLOCK) rowf[s] = 0;
        for (uint32_t s = threadIdx.x; s < ncols; s += BLOCK) colf[s] = 0;
    }
    __syncthreads();

    const float* src = w + T.offset + e0;
    float* dst = FUSED ? w_out + T.offset + e0 : nullptr;
    uint8_t* mdst = (FUSED && T.prunable && mask) ? mask + T.gbase + e0 : nullptr;
    uint32_t below = 0, nan = 0;

    // classifies one weight: returns the bits to store, sets keep / is_cand
    auto one = [&](uint32_t j, uint32_t bits, uint32_t& keep, bool& is_cand) -> uint32_t {
        const uint32_t key = bits & 0x7fffffffu;
        const bool removed = ranked && key < mid;       // lo <= mid <= hi
        is_cand = ranked && key >= lo && key <= hi;
        below += (ranked && key < lo) ? 1u : 0u;
        nan |= (ranked && key > 0x7f800000u) ? 1u : 0u;
        keep = removed ? 0u : 1u;
        if (FUSED && !removed && !is_cand && key != 0) {
            rowf[div_small(r0 + j, T.row_len, T.magic_row)] = 1;
            colf[div_small(c0 + j, T.khw, T.magic_khw)] = 1;
        }
        return removed ? 0u : bits;
    };

    const bool vec_ok = n == TILE && (T.offset & 3u) == 0 && (!mdst || (T.gbase & 3u) == 0);
    if (vec_ok) {
        constexpr uint32_t U = TILE / BLOCK / 4;
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
        uint4 v[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) v[u] = load_u4<NT>(s4 + threadIdx.x + BLOCK * u);
        uint32_t cmask = 0;
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = (threadIdx.x + BLOCK * u) * 4;
            uint32_t k0, k1, k2, k3;
            bool q0, q1, q2, q3;
            uint4 o;
            o.x = one(j, v[u].x, k0, q0);
            o.y = one(j + 1, v[u].y, k1, q1);
            o.z = one(j + 2, v[u].z, k2, q2);
            o.w = one(j + 3, v[u].w, k3, q3);
            cmask |= ((q0 ? 1u : 0u) | (q1 ? 2u : 0u) | (q2 ? 4u : 0u) | (q3 ? 8u : 0u)) << (4 * u);
            if (FUSED) {
                store_u4<NT>(reinterpret_cast<uint4*>(dst) + threadIdx.x + BLOCK * u, o);
                if (mdst)
                    store_u1<NT>(reinterpret_cast<uint32_t*>(mdst) + threadIdx.x + BLOCK * u,
                                 k0 | (k1 << 8) | (k2 << 16) | (k3 << 24));
            }
        }
        // append the block's candidates with one global atomic: scan the per-thread
        // counts over the block, reserve a range in this block's sub-buffer, scatter
        const uint32_t c = __popc(cmask);
        uint32_t incl = c;
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(incl, d, 64);
            if (lane >= d) incl += y;
        }
        if (lane == 63) s_wtot[wid] = incl;
        __syncthreads();
        uint32_t woff = 0, btot = 0;
#pragma unroll
        for (uint32_t i = 0; i < BLOCK / 64; ++i) {
            const uint32_t x = s_wtot[i];
            if (i < wid) woff += x;
            btot += x;
        }
        if (btot) {   // uniform over the block
            if (threadIdx.x == 0) s_base = atomicAdd(sub_counter(cnt, CNT_CAND, sb), btot);
            __syncthreads();
            uint32_t pos = s_base + woff + incl - c;
            if (cmask) {
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    const uint32_t j = (threadIdx.x + BLOCK * u) * 4;
                    const uint32_t vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                    for (uint32_t q = 0; q < 4; ++q) {
                        if (cmask & (1u << (4 * u + q))) {
                            if (pos < cap_sb)
                                my_cand[pos] = make_uint2(vv[q], g0 + j + q);
                            ++pos;
                        }
                    }
                }
            }
        }
    } else {
        // ragged or unaligned tile (at most a few per tensor): one atomic per candidate
        for (uint32_t j = threadIdx.x; j < n; j += BLOCK) {
            uint32_t k;
            bool q;
            const uint32_t bits = __float_as_uint(src[j]);
            const uint32_t o = one(j, bits, k, q);
            if (FUSED) {
                dst[j] = __uint_as_float(o);
                if (mdst) mdst[j] = (uint8_t)k;
            }
            if (q) {
                const uint32_t pos = atomicAdd(sub_counter(cnt, CNT_CAND, sb), 1u);
                if (pos < cap_sb) my_cand[pos] = make_uint2(bits, g0 + j);
            }
        }
    }
    for (uint32_t d = 32; d > 0; d >>= 1) {
        below += __shfl_down(below, d, 64);
        nan |= __shfl_down(nan, d, 64);
    }
    if (lane == 0) {
        if (below) atomicAdd(&s_below, below);
        if (nan) s_nan = 1;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (s_below) atomicAdd(sub_counter(cnt, CNT_BELOW, sb), s_below);
        if (s_nan) atomicOr(&ss->status, 2u);
    }
    if (FUSED) {
        const uint32_t row_first = e0 / T.row_len;
        for (uint32_t s = threadIdx.x; s < nrows; s += BLOCK) {
            if (rowf[s]) {
                uint8_t* f = out_alive + T.out_flag_off + row_first + s;
                if (*f == 0) *f = 1;
            }
        }
        const uint32_t b = (e0 / T.khw) % T.in_ch;
        for (uint32_t s = threadIdx.x; s < ncols; s += BLOCK) {
            if (colf[s]) {
                uint8_t* f = in_alive + T.in_flag_off + mod_small(b + s, T.in_ch, T.magic_in);
                if (*f == 0) *f = 1;
            }
        }
    }
}

// Visits every candidate pair.  The grid is a multiple of SPEC_SUB blocks: block b walks
// sub-buffer b % SPEC_SUB, taking every (gridDim / SPEC_SUB)-th chunk of BLOCK pairs.
// Every thread of the block calls f the same number of times; `valid` is false for the
// threads past the end of the last, ragged chunk.
template <typename F>
__device__ __forceinline__ void for_each_candidate(const uint32_t* cnt, const uint2* cand,
                                                   uint32_t cap_sb, F&& f) {
    const uint32_t sb = blockIdx.x % SPEC_SUB, part = blockIdx.x / SPEC_SUB;
    const uint32_t parts = gridDim.x / SPEC_SUB;
    const uint32_t n = min(cnt[(CNT_CAND * SPEC_SUB + sb) * 32u], cap_sb);
    const uint2* src = cand + (size_t)sb * cap_sb;
    // four chunks per step: the loads of a step are all in flight before the first is used
    // (a block holds few wavefronts, so one load per thread at a time leaves the walk
    // waiting on memory latency)
    constexpr uint32_t U = 4;
    for (uint32_t i0 = part * BLOCK; i0 < n; i0 += U * parts * BLOCK) {
        uint2 c[U];
        bool valid[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t i = i0 + u * parts * BLOCK + threadIdx.x;
            valid[u] = i < n;
            c[u] = valid[u] ? src[i] : make_uint2(0, 0);
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) f(c[u], valid[u]);
    }
}

// Totals of the split counters, the check that makes the result exact, then the round-1
// bin holding the P-th pair.  Every block of the filter kernel runs this on the same
// inputs (64 KB of partial histograms from L2) and gets the same answer, which is cheaper
// than a kernel of its own or a fenced rendezvous; `publish` is set for one block, which
// records the outcome.  Returns false when the single pass cannot decide.
__device__ bool spec_locate(SpecState* ss, const uint32_t* __restrict__ cnt,
                            const uint32_t* __restrict__ partial, uint32_t cap_sb,
                            uint64_t* smem, bool publish, uint32_t* bin_out) {
    __shared__ uint32_t s_over;
    const uint64_t p = ss->p;
    if (threadIdx.x == 0) s_over = 0;
    __syncthreads();
    uint64_t below = 0, inside = 0, tot;
    static_assert(SPEC_SUB == BLOCK, "one split counter per thread");
    {
        const uint32_t c = cnt[(CNT_CAND * SPEC_SUB + threadIdx.x) * 32u];
        const uint32_t b = cnt[(CNT_BELOW * SPEC_SUB + threadIdx.x) * 32u];
        block_excl_scan_u64(c, smem, &inside);
        block_excl_scan_u64(b, smem, &below);
        if (c > cap_sb) s_over = 1;
    }
    __syncthreads();
    if (publish && threadIdx.x == 0) { ss->n_below = below; ss->n_inside = inside; }
    if (s_over || !(below < p && p <= below + inside)) {
        if (publish && threadIdx.x == 0) atomicOr(&ss->status, 1u);
        return false;
    }
    const uint64_t r = p - below;
    static_assert(FBINS1 == BLOCK, "one round-1 bin per thread");
    // sum the FIN_BLOCKS partial histograms: thread t reads the uint4s t, t + 256, ...;
    // each covers the same four bins (4t mod 256 ...), so it keeps four sums and four
    // threads then meet in LDS.  All loads are independent of each other.
    __shared__ uint32_t s_bins[FBINS1];
    s_bins[threadIdx.x] = 0;
    __syncthreads();
    {
        const uint4* p4 = reinterpret_cast<const uint4*>(partial);
        uint4 acc = make_uint4(0, 0, 0, 0);
        constexpr uint32_t N4 = FIN_BLOCKS * FBINS1 / 4 / BLOCK;
#pragma unroll 16
        for (uint32_t i = 0; i < N4; ++i) {
            const uint4 x = p4[threadIdx.x + BLOCK * i];
            acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
        }
        const uint32_t b4 = (4u * threadIdx.x) & (FBINS1 - 1);
        atomicAdd(&s_bins[b4], acc.x);
        atomicAdd(&s_bins[b4 + 1], acc.y);
        atomicAdd(&s_bins[b4 + 2], acc.z);
        atomicAdd(&s_bins[b4 + 3], acc.w);
    }
    __syncthreads();
    const uint32_t c = s_bins[threadIdx.x];
    const uint64_t base = block_excl_scan_u64(c, smem, &tot);
    __shared__ uint32_t s_bin, s_ok;
    if (base < r && r <= base + c) {
        s_bin = threadIdx.x;
        s_ok = c <= SPEC_LIST_CAP ? 1u : 0u;
        if (publish) {
            ss->bin = threadIdx.x;
            ss->bin_cnt = c;
            ss->r2 = r - base;
            ss->less = below + base;
            if (c > SPEC_LIST_CAP) atomicOr(&ss->status, 1u);
        }
    }
    __syncthreads();
    *bin_out = s_bin;
    return s_ok != 0;
}

// Round 1: per-block LDS histogram of (key - lo) >> sh (256 bins) over the candidates; the
// partial histograms go to global memory side by side (no atomics).
__global__ __launch_bounds__(BLOCK) void spec_hist_kernel(const SpecState* __restrict__ ss,
                                                          const uint32_t* __restrict__ cnt,
                                                          const uint2* __restrict__ cand,
                                                          uint32_t cap_sb,
                                                          uint32_t* __restrict__ partial) {
    __shared__ uint32_t h[FBINS1];
    h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t lo = ss->lo, sh = ss->sh;
    for_each_candidate(cnt, cand, cap_sb, [&](uint2 c, bool valid) {
        if (valid) atomicAdd(&h[((c.x & 0x7fffffffu) - lo) >> sh], 1u);
    });
    __syncthreads();
    partial[blockIdx.x * FBINS1 + threadIdx.x] = h[threadIdx.x];
}

// One block: round-2 histogram over the list, then an exact rank (by counting) among the
// pairs of the selected round-2 bin, then the record.
// Whatever the outcome, the state (status, counts, the record) is left in its mirror in
// pinned host memory as the last thing: the host reads it after waiting for the stream,
// with no copy on the stream.
__global__ __launch_bounds__(BLOCK) void spec_rank_kernel(SpecState* ss,
                                                          const uint2* __restrict__ list,
                                                          shifter_threshold* thr, SpecState* host_mirror) {
    // only thread 0 writes the state in this kernel, so it reads back its own writes
    auto publish = [&]() {
        if (threadIdx.x == 0) *host_mirror = *ss;
    };
    __shared__ uint32_t h[FBINS];
    __shared__ uint64_t comp[SPEC_SMALL_CAP];
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint64_t s_sel, s_less2, s_r3;
    __shared__ uint32_t s_lt, s_eq, s_bin2, s_cnt2, s_nb;
    shifter_threshold out;
    out.reserved = 0;
    out.n_prune = ss->p;
    if (ss->p == 0) {
        if (threadIdx.x == 0) {
            out.cut = 0; out.t_key = 0; out.g_cut = ~0ull; out.n_less = 0; out.n_equal = 0;
            *thr = out;
            ss->rec = out;
        }
        publish();
        return;
    }
    // Undecided: the host redoes the ranking and every step behind it.  What is enqueued
    // behind this kernel still runs once on the record it finds, so leave a harmless one
    // (nothing removed) rather than the record of some earlier call.
    auto undecided = [&]() {
        if (threadIdx.x == 0) {
            out.cut = 0; out.t_key = 0; out.g_cut = ~0ull; out.n_less = 0; out.n_equal = 0;
            *thr = out;
        }
        publish();
    };
    if (ss->status & 1u) { undecided(); return; }
    const uint32_t n = min(ss->list_cnt, SPEC_LIST_CAP);
    if (n != ss->bin_cnt) {   // cannot happen unless the buffers were disturbed
        if (threadIdx.x == 0) atomicOr(&ss->status, 1u);
        undecided();
        return;
    }
    // round 2: the list's keys span 2^sh values starting at lo + (bin << sh)
    const uint32_t sh = ss->sh;
    const uint32_t sh2 = sh > 12 ? sh - 12 : 0;   // 2^sh keys over FBINS = 2^12 bins
    const uint32_t lo1 = ss->lo + (ss->bin << sh);
    for (uint32_t i = threadIdx.x; i < FBINS; i += BLOCK) h[i] = 0;
    if (threadIdx.x == 0) { s_lt = 0; s_eq = 0; s_sel = 0; s_nb = 0; s_cnt2 = 0; s_bin2 = 0; }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK)
        atomicAdd(&h[((list[i].x & 0x7fffffffu) - lo1) >> sh2], 1u);
    __syncthreads();
    constexpr uint32_t PER = FBINS / BLOCK;
    const uint32_t b0 = threadIdx.x * PER;
    uint64_t sum = 0, tot;
    for (uint32_t i = 0; i < PER; ++i) sum += h[b0 + i];
    uint64_t base = block_excl_scan_u64(sum, smem, &tot);
    const uint64_t r = ss->r2;
    if (base < r && r <= base + sum) {
        for (uint32_t i = 0; i < PER; ++i) {
            const uint32_t c = h[b0 + i];
            if (r <= base + c) {
                s_bin2 = b0 + i;
                s_cnt2 = c;
                s_r3 = r - base;
                s_less2 = base;
                break;
            }
            base += c;
        }
    }
    __syncthreads();
    const uint32_t bin2 = s_bin2, cnt2 = s_cnt2;
    if (cnt2 == 0 || cnt2 > SPEC_SMALL_CAP) {
        if (threadIdx.x == 0) atomicOr(&ss->status, 1u);
        undecided();
        return;
    }
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) {
        const uint2 c = list[i];
        const uint32_t key = c.x & 0x7fffffffu;
        if (((key - lo1) >> sh2) == bin2) {
            const uint32_t pos = atomicAdd(&s_nb, 1u);
            comp[pos] = ((uint64_t)key << 32) | c.y;   // pos < cnt2 <= SPEC_SMALL_CAP
        }
    }
    __syncthreads();
    const uint64_t want = s_r3 - 1;   // 0-based rank inside the bin
    for (uint32_t i = threadIdx.x; i < cnt2; i += BLOCK) {
        const uint64_t c = comp[i];
        uint32_t rank = 0;
        for (uint32_t f = 0; f < cnt2; ++f) rank += comp[f] < c;
        if (rank == want) s_sel = c;    // composites are distinct: exactly one hit
    }
    __syncthreads();
    const uint64_t sel = s_sel;
    const uint32_t key = (uint32_t)(sel >> 32);
    uint32_t lt = 0, eq = 0;
    for (uint32_t i = threadIdx.x; i < cnt2; i += BLOCK) {
        const uint32_t k = (uint32_t)(comp[i] >> 32);
        lt += k < key;
        eq += k == key;
    }
    if (lt) atomicAdd(&s_lt, lt);
    if (eq) atomicAdd(&s_eq, eq);
    __syncthreads();
    if (threadIdx.x == 0) {
        out.t_key = key;
        out.g_cut = sel & 0xffffffffull;
        out.cut = sel + 1;
        out.n_less = ss->less + s_less2 + s_lt;
        out.n_equal = s_eq;
        *thr = out;
        ss->rec = out;
    }
    publish();
}

// Candidates of the selected round-1 bin -> list.  Each block stages its hits in LDS and
// reserves its range of the list with one global atomic.
__global__ __launch_bounds__(BLOCK) void spec_filter_kernel(SpecState* ss,
                                                            const uint32_t* __restrict__ cnt,
                                                            const uint32_t* __restrict__ partial,
                                                            const uint2* __restrict__ cand,
                                                            uint32_t cap_sb, uint2* list) {
    constexpr uint32_t STAGE = 2048;
    __shared__ uint2 stage[STAGE];
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t s_n, s_base;
    if (ss->p == 0) return;
    uint32_t bin;
    if (threadIdx.x == 0) s_n = 0;
    if (!spec_locate(ss, cnt, partial, cap_sb, smem, blockIdx.x == 0, &bin)) return;
    const uint32_t lo = ss->lo, sh = ss->sh;
    for_each_candidate(cnt, cand, cap_sb, [&](uint2 c, bool valid) {
        if (valid && (((c.x & 0x7fffffffu) - lo) >> sh) == bin) {
            const uint32_t pos = atomicAdd(&s_n, 1u);
            if (pos < STAGE) stage[pos] = c;
        }
    });
    __syncthreads();
    const uint32_t n = s_n;
    if (n > STAGE) {   // far more ties than the stage holds: leave it to the radix select
        if (threadIdx.x == 0) atomicOr(&ss->status, 1u);
        return;
    }
    if (n == 0) return;
    if (threadIdx.x == 0) s_base = atomicAdd(&ss->list_cnt, n);
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK)
        if (s_base + i < SPEC_LIST_CAP) list[s_base + i] = stage[i];
}

// Fused form only: settle the candidates.  The pass wrote those below mid as removed and
// the others as kept without flags; with the exact cut known, the few on the wrong side
// are rewritten and every kept non-zero candidate marks its filter and input feature.
__global__ __launch_bounds__(BLOCK) void spec_fixup_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ ranked_ids,
    uint32_t n_ranked, const SpecState* __restrict__ ss, const uint32_t* __restrict__ cnt,
    const uint2* __restrict__ cand, uint32_t cap_sb, const shifter_threshold* __restrict__ thr,
    float* __restrict__ w_out, uint8_t* __restrict__ mask, uint8_t* out_alive,
    uint8_t* in_alive) {
    constexpr uint32_t LDS_T = 1024;
    __shared__ uint32_t s_gbase[LDS_T];
    if (ss->p == 0 || (ss->status & 1u)) return;
    const uint64_t cut = thr->cut;
    const uint32_t mid = ss->mid;
    const bool in_lds = n_ranked <= LDS_T;
    if (in_lds)
        for (uint32_t i = threadIdx.x; i < n_ranked; i += BLOCK)
            s_gbase[i] = (uint32_t)tens[ranked_ids[i]].gbase;
    __syncthreads();
    for_each_candidate(cnt, cand, cap_sb, [&](uint2 c, bool valid) {
        if (!valid) return;
        const uint32_t key = c.x & 0x7fffffffu;
        const bool removed = (((uint64_t)key << 32) | c.y) < cut;
        const bool written_removed = key < mid;
        if (removed == written_removed && (removed || key == 0)) return;   // nothing to do
        // tensor holding global index c.y: last ranked tensor with gbase <= g
        uint32_t a = 0, b = n_ranked;
        while (b - a > 1) {
            const uint32_t m2 = (a + b) >> 1;
            const uint32_t gb = in_lds ? s_gbase[m2] : (uint32_t)tens[ranked_ids[m2]].gbase;
            if (gb <= c.y) a = m2; else b = m2;
        }
        const DevTensor& T = tens[ranked_ids[a]];
        const uint32_t e = c.y - (uint32_t)T.gbase;
        if (removed != written_removed) {
            w_out[T.offset + e] = removed ? 0.0f : __uint_as_float(c.x);
            if (mask) mask[c.y] = removed ? 0 : 1;
        }
        if (!removed && key != 0) {
            uint8_t* f = out_alive + T.out_flag_off + e / T.row_len;
            if (*f == 0) *f = 1;
            f = in_alive + T.in_flag_off + (e / T.khw) % T.in_ch;
            if (*f == 0) *f = 1;
        }
    });
}

void launch_spec_sample(shifter_ctx* ctx, const shifter_model* m, const float* d_w, const SampleZero& z) {
    const auto& b = m->b;
    const uint32_t sampled = (m->n_tiles + m->sample_tile_stride - 1) / m->sample_tile_stride;
    // one block per CU: more blocks shorten the loop but every block flushes its LDS
    // histogram with global atomics (measured with 256-thread blocks: 22 us at 256 blocks,
    // 24 at 512, 34 at 128 or 1024; 1024-thread blocks brought the 256 to 15 us)
    const uint32_t grid = std::min(256u, (sampled + 63) / 64);   // 64 tiles per block and step
    spec_sample_kernel<<<grid, SAMPLE_THREADS, 0, ctx->stream>>>(b.tens, b.tile_prefix, b.tile_tensor,
                                                        m->n_tiles, m->sample_tile_stride, d_w,
                                                        b.shist, z);
}

void launch_spec_select(shifter_ctx* ctx, const shifter_model* m, const float* d_w, uint64_t p,
                        shifter_threshold* d_thr, float* d_w_out, uint8_t* d_mask,
                        uint8_t* d_out_alive, uint8_t* d_in_alive, SpecState* host_mirror) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size();
    const bool fused = d_w_out != nullptr;
    hipStream_t s = ctx->stream;
    {
        // the set-up rides on the sample kernel
        ProfileScope ps(ctx, K_SPEC_SAMPLE);
        SampleZero z;
        z.ss = b.spec;
        z.cnt1 = b.spec_cnt;
        z.p = p;
        z.m_valid = m->sample_size;
        z.fa = d_out_alive;
        z.na = fused ? m->info.sum_out_ch : 0;
        z.fb = d_in_alive;
        z.nb = fused ? m->info.sum_in_ch : 0;
        launch_spec_sample(ctx, m, d_w, z);
    }
    {
        ProfileScope ps(ctx, K_SPEC_PREDICT);
        spec_predict_kernel<<<1, BLOCK, 0, s>>>(b.spec, b.shist, m->info.n_prunable,
                                                ctx->margin_sigmas);
    }
    {
        ProfileScope ps(ctx, K_SPEC_PASS);
        const bool nt = m->info.w_extent * 4 > (192ull << 20);   // beyond the last-level cache
        auto k = fused ? (nt ? spec_pass_kernel<true, true> : spec_pass_kernel<true, false>)
                       : (nt ? spec_pass_kernel<false, true> : spec_pass_kernel<false, false>);
        k<<<m->n_tiles, BLOCK, 0, s>>>(b.tens, b.tile_prefix, n_t, d_w, b.spec, b.spec_cnt, b.cand,
                                       b.cand_cap_sb, d_w_out, d_mask, d_out_alive, d_in_alive);
    }
    {
        ProfileScope ps(ctx, K_SPEC_FINISH);
        spec_hist_kernel<<<FIN_BLOCKS, BLOCK, 0, s>>>(b.spec, b.spec_cnt, b.cand, b.cand_cap_sb,
                                                      b.partial);
    }
    {
        ProfileScope ps(ctx, K_SPEC_FINISH2);
        spec_filter_kernel<<<FIN_BLOCKS, BLOCK, 0, s>>>(b.spec, b.spec_cnt, b.partial, b.cand,
                                                        b.cand_cap_sb, b.list);
        spec_rank_kernel<<<1, BLOCK, 0, s>>>(b.spec, b.list, d_thr, host_mirror);
    }
    if (fused) {
        ProfileScope ps(ctx, K_SPEC_FIXUP);
        spec_fixup_kernel<<<SPEC_SUB * 4, BLOCK, 0, s>>>(
            b.tens, b.ranked_ids, m->n_ranked, b.spec, b.spec_cnt, b.cand, b.cand_cap_sb, d_thr,
            d_w_out, d_mask, d_out_alive, d_in_alive);
    }
}

}  // namespace shifter
