// Single-pass exact selection for ALL prune counts of a portfolio at once: the ranking of
// Sec. II-A / Sec. III-C of the paper for K sparsity levels in one read of the arena.
//
// Same scheme as the one-count selection (sample, predict, one pass, finish), with the
// prune counts sorted ascending so that the predicted key intervals [lo_k, hi_k] have
// non-decreasing ends.  For a weight with key x let j = #{k : lo_k <= x}; then
//   x < lo_k  <=>  j <= k            (so below_k is a prefix sum of the counts per j)
//   x is a candidate of some rank  <=>  j >= 1 and x <= hi_{j-1}
//   x is a candidate of rank k  <=>  first{k : hi_k >= x} <= k < j
// so one binary search per weight replaces K interval tests.  The candidates of all
// ranks share the 256 sub-buffers; the finishing passes visit each candidate once and
// update every rank whose interval holds it.
#include "dev_common.h"

namespace shifter {

constexpr uint32_t MS_BINS = 16384;      // sample histogram bins
constexpr uint32_t MS_SHIFT = 17;        // top 14 of the 31 key bits
constexpr uint32_t MF_BINS1 = 256;       // round-1 finishing histogram, per rank
constexpr uint32_t MF_BINS2 = 4096;      // round-2, one block per rank
constexpr uint32_t MF_BLOCKS = SPEC_SUB; // blocks of the passes over the candidates

enum { MC_CAND = 0, MC_BELOW = 1 };   // cnt layout: [MC_CAND][sb]*32, then [1 + j][sb]*32

__device__ __forceinline__ uint32_t* mcnt(uint32_t* cnt, uint32_t which, uint32_t sb) {
    return cnt + ((size_t)which * SPEC_SUB + sb) * 32u;
}

// sorted_p / perm: the k prune counts > 0 in ascending order and their original positions;
// zero_mask: bit i set = original position i asked for P = 0 and gets its record here.
__global__ __launch_bounds__(BLOCK) void ms_init_kernel(MultiState* ms, uint32_t* shist,
                                                        uint32_t* cnt, PruneCounts sorted_p,
                                                        MultiPerm perm, uint32_t k,
                                                        uint32_t m_valid, uint64_t zero_mask,
                                                        shifter_threshold* thr) {
    const uint64_t tid = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * BLOCK;
    for (uint64_t i = tid; i < MS_BINS; i += stride) shist[i] = 0;
    for (uint64_t i = tid; i < (uint64_t)(k + 2) * SPEC_SUB * 32u; i += stride) cnt[i] = 0;
    if (tid < MAXK) {
        ms->p[tid] = tid < k ? sorted_p.p[tid] : 0;
        ms->perm[tid] = tid < k ? perm.v[tid] : 0;
        ms->lo[tid] = 0xffffffffu;     // padding sorts last in the searches
        ms->hi[tid] = 0xffffffffu;
        ms->sh[tid] = 0;
        ms->bin[tid] = 0;
        ms->bin_cnt[tid] = 0;
        ms->r2[tid] = 0;
        ms->less[tid] = 0;
    }
    if (tid < MAXK && ((zero_mask >> tid) & 1ull)) {
        shifter_threshold out;
        out.cut = 0; out.t_key = 0; out.reserved = 0; out.g_cut = ~0ull; out.n_prune = 0;
        out.n_less = 0; out.n_equal = 0;
        thr[tid] = out;
    }
    if (tid == 0) {
        ms->k = k;
        ms->m_valid = m_valid;
        ms->status = 0;
    }
}

// One block: inclusive prefix of the sample histogram in LDS, then for every rank the
// interval from the sample's order statistics at P/N -/+ margin, then monotone ends.
__global__ __launch_bounds__(BLOCK) void ms_predict_kernel(MultiState* ms,
                                                           const uint32_t* __restrict__ shist,
                                                           uint64_t n_prunable,
                                                           double margin_sigmas) {
    constexpr uint32_t SEG = 256, NSEG = MS_BINS / SEG;
    __shared__ uint32_t prefix[MS_BINS];          // 64 KB
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t seg_sum[NSEG];
    __shared__ uint32_t s_lo[MAXK], s_hi[MAXK];
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    // phase 1: segment sums
    for (uint32_t sg = wid; sg < NSEG; sg += BLOCK / 64) {
        const uint4 x = reinterpret_cast<const uint4*>(shist + sg * SEG)[lane];
        uint32_t v = x.x + x.y + x.z + x.w;
        for (uint32_t d = 32; d > 0; d >>= 1) v += __shfl_down(v, d, 64);
        if (lane == 0) seg_sum[sg] = v;
    }
    __syncthreads();
    const uint64_t mine = threadIdx.x < NSEG ? seg_sum[threadIdx.x] : 0;
    uint64_t total;
    const uint64_t base = block_excl_scan_u64(mine, smem, &total);
    if (threadIdx.x < NSEG) seg_sum[threadIdx.x] = (uint32_t)base;   // exclusive segment base
    __syncthreads();
    // phase 2: inclusive prefix per bin
    for (uint32_t sg = wid; sg < NSEG; sg += BLOCK / 64) {
        const uint4 x = reinterpret_cast<const uint4*>(shist + sg * SEG)[lane];
        const uint32_t mine4 = x.x + x.y + x.z + x.w;
        uint32_t incl = mine4;
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(incl, d, 64);
            if (lane >= d) incl += y;
        }
        uint32_t run = seg_sum[sg] + incl - mine4;
        uint32_t* out = prefix + sg * SEG + lane * 4;
        run += x.x; out[0] = run;
        run += x.y; out[1] = run;
        run += x.z; out[2] = run;
        run += x.w; out[3] = run;
    }
    __syncthreads();
    const uint32_t k_var = ms->k;
    const uint32_t m = ms->m_valid;
    if (threadIdx.x < k_var) {
        const uint64_t p = ms->p[threadIdx.x];
        uint32_t lo = 0, hi = 0x7fffffffu;
        if (p > 0 && m >= 256 && n_prunable > 0 && total == m) {
            const double frac = (double)p / (double)n_prunable;
            const double centre = frac * (double)m;
            const double delta = margin_sigmas * sqrt((double)m * frac * (1.0 - frac)) + 16.0;
            auto bin_of = [&](double r) -> uint32_t {   // first bin with prefix > r
                const uint32_t target = (uint32_t)r;
                uint32_t a = 0, b = MS_BINS - 1;
                while (a < b) {
                    const uint32_t mid = (a + b) >> 1;
                    if (prefix[mid] > target) b = mid; else a = mid + 1;
                }
                return a;
            };
            const double r_lo = centre - delta, r_hi = centre + delta;
            if (r_lo > 0.0) lo = bin_of(r_lo) << MS_SHIFT;
            if (r_hi < (double)(m - 1)) hi = ((bin_of(r_hi) + 1u) << MS_SHIFT) - 1u;
        }
        s_lo[threadIdx.x] = lo;
        s_hi[threadIdx.x] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        // widen so that both ends are non-decreasing in k (ranks are sorted by P)
        for (uint32_t k = 1; k < k_var; ++k) s_hi[k] = max(s_hi[k], s_hi[k - 1]);
        for (uint32_t k = k_var - 1; k > 0; --k) s_lo[k - 1] = min(s_lo[k - 1], s_lo[k]);
        for (uint32_t k = 0; k < k_var; ++k) {
            uint32_t sh = 0;
            while (((s_hi[k] - s_lo[k]) >> sh) >= MF_BINS1) ++sh;
            ms->lo[k] = s_lo[k];
            ms->hi[k] = s_hi[k];
            ms->sh[k] = sh;
        }
    }
}

// The one pass over the arena: counts per j and candidate pairs.
template <bool NT>
__global__ __launch_bounds__(BLOCK) void ms_pass_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix, uint32_t n_t,
    const float* __restrict__ w, MultiState* ms, uint32_t* cnt, uint2* __restrict__ cand,
    uint32_t cap_sb) {
    __shared__ uint32_t s_lo[MAXK + 1], s_hi[MAXK + 1];
    // counts per j: one private column per thread (no conflicts, no atomics), summed at
    // the end; rows 0 .. k_var
    __shared__ uint32_t s_col[(SPEC_MULTI_MAXK + 1) * BLOCK];
    __shared__ uint32_t s_nan, s_base, s_wtot[BLOCK / 64];
    const uint32_t tile = blockIdx.x;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    if (!tens[t].prunable) return;
    const DevTensor T = tens[t];
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const uint32_t g0 = (uint32_t)(T.gbase + e0);
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    const uint32_t sb = blockIdx.x & (SPEC_SUB - 1);
    uint2* my_cand = cand + (size_t)sb * cap_sb;
    const uint32_t k_var = ms->k;
    if (threadIdx.x <= MAXK) {
        s_lo[threadIdx.x] = threadIdx.x < MAXK ? ms->lo[threadIdx.x] : 0xffffffffu;
        s_hi[threadIdx.x] = threadIdx.x < MAXK ? ms->hi[threadIdx.x] : 0xffffffffu;
    }
    for (uint32_t j = 0; j <= k_var; ++j) s_col[j * BLOCK + threadIdx.x] = 0;
    if (threadIdx.x == 0) { s_nan = 0; s_base = 0; }
    __syncthreads();

    uint32_t nan = 0;
    // classify one weight; returns whether it is a candidate; adds it to the count of j
    auto one = [&](uint32_t bits) -> bool {
        const uint32_t key = bits & 0x7fffffffu;
        nan |= key > 0x7f800000u ? 1u : 0u;
        uint32_t j = 0;
#pragma unroll
        for (uint32_t step = MAXK / 2; step >= 1; step >>= 1)
            if (s_lo[j + step - 1] <= key) j += step;
        j += s_lo[j] <= key ? 1u : 0u;          // j in [0, MAXK]; s_lo[MAXK] is padding
        const bool is_cand = j >= 1 && key <= s_hi[j - 1];
        s_col[j * BLOCK + threadIdx.x] += 1;    // j <= k_var <= SPEC_MULTI_MAXK
        return is_cand;
    };

    const float* src = w + T.offset + e0;
    if (n == TILE && (T.offset & 3u) == 0) {
        constexpr uint32_t U = TILE / BLOCK / 4;
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
        uint4 v[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) v[u] = load_u4<NT>(s4 + threadIdx.x + BLOCK * u);
        uint32_t cmask = 0;
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            cmask |= ((one(v[u].x) ? 1u : 0u) | (one(v[u].y) ? 2u : 0u) | (one(v[u].z) ? 4u : 0u) |
                      (one(v[u].w) ? 8u : 0u)) << (4 * u);
        }
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
            if (threadIdx.x == 0) s_base = atomicAdd(mcnt(cnt, MC_CAND, sb), btot);
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
                            if (pos < cap_sb) my_cand[pos] = make_uint2(vv[q], g0 + j + q);
                            ++pos;
                        }
                    }
                }
            }
        }
    } else {
        for (uint32_t j0 = 0; j0 < n; j0 += BLOCK) {
            const uint32_t j = j0 + threadIdx.x;
            if (j < n) {
                const uint32_t bits = __float_as_uint(src[j]);
                if (one(bits)) {
                    const uint32_t pos = atomicAdd(mcnt(cnt, MC_CAND, sb), 1u);
                    if (pos < cap_sb) my_cand[pos] = make_uint2(bits, g0 + j);
                }
            }
        }
    }
    for (uint32_t d = 32; d > 0; d >>= 1) nan |= __shfl_down(nan, d, 64);
    if (lane == 0 && nan) s_nan = 1;
    __syncthreads();
    // column sums: four threads per j, a quarter of the columns each
    if (threadIdx.x < 4 * (k_var + 1)) {
        const uint32_t j = threadIdx.x >> 2, q = threadIdx.x & 3u;
        uint32_t c = 0;
        for (uint32_t i = 0; i < BLOCK / 4; ++i) c += s_col[j * BLOCK + ((i * 4 + q + j) & (BLOCK - 1))];
        if (c) atomicAdd(mcnt(cnt, MC_BELOW + j, sb), c);
    }
    if (threadIdx.x == 0 && s_nan) atomicOr(&ms->status, 2u);
}

// Visits every candidate pair (see the one-count selection).
template <typename F>
__device__ __forceinline__ void ms_for_each_candidate(const uint32_t* cnt, const uint2* cand,
                                                      uint32_t cap_sb, F&& f) {
    const uint32_t sb = blockIdx.x % SPEC_SUB, part = blockIdx.x / SPEC_SUB;
    const uint32_t parts = gridDim.x / SPEC_SUB;
    const uint32_t n = min(cnt[((size_t)MC_CAND * SPEC_SUB + sb) * 32u], cap_sb);
    const uint2* src = cand + (size_t)sb * cap_sb;
    for (uint32_t i0 = part * BLOCK; i0 < n; i0 += parts * BLOCK) {
        const uint32_t i = i0 + threadIdx.x;
        const bool valid = i < n;
        f(valid ? src[i] : make_uint2(0, 0), valid);
    }
}

// ranks whose interval holds key: [ka, kb)
__device__ __forceinline__ void rank_range(const uint32_t* s_lo, const uint32_t* s_hi, uint32_t key,
                                           uint32_t* ka, uint32_t* kb) {
    uint32_t j = 0, a = 0;
#pragma unroll
    for (uint32_t step = MAXK / 2; step >= 1; step >>= 1) {
        if (s_lo[j + step - 1] <= key) j += step;
        if (s_hi[a + step - 1] < key) a += step;
    }
    j += s_lo[j] <= key ? 1u : 0u;
    a += s_hi[a] < key ? 1u : 0u;
    *ka = a;   // first k with hi_k >= key
    *kb = j;   // #{k : lo_k <= key}
}

// Round 1: per block and per rank a 256-bin LDS histogram of (key - lo_k) >> sh_k.
__global__ __launch_bounds__(BLOCK) void ms_hist_kernel(const MultiState* __restrict__ ms,
                                                        const uint32_t* __restrict__ cnt,
                                                        const uint2* __restrict__ cand,
                                                        uint32_t cap_sb,
                                                        uint32_t* __restrict__ partial) {
    extern __shared__ uint32_t h[];   // k_var * 256
    __shared__ uint32_t s_lo[MAXK + 1], s_hi[MAXK + 1], s_sh[MAXK];
    const uint32_t k_var = ms->k;
    for (uint32_t i = threadIdx.x; i < k_var * MF_BINS1; i += BLOCK) h[i] = 0;
    if (threadIdx.x <= MAXK) {
        s_lo[threadIdx.x] = threadIdx.x < MAXK ? ms->lo[threadIdx.x] : 0xffffffffu;
        s_hi[threadIdx.x] = threadIdx.x < MAXK ? ms->hi[threadIdx.x] : 0xffffffffu;
        if (threadIdx.x < MAXK) s_sh[threadIdx.x] = ms->sh[threadIdx.x];
    }
    __syncthreads();
    ms_for_each_candidate(cnt, cand, cap_sb, [&](uint2 c, bool valid) {
        if (!valid) return;
        const uint32_t key = c.x & 0x7fffffffu;
        uint32_t ka, kb;
        rank_range(s_lo, s_hi, key, &ka, &kb);
        for (uint32_t k = ka; k < kb; ++k)
            atomicAdd(&h[k * MF_BINS1 + ((key - s_lo[k]) >> s_sh[k])], 1u);
    });
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < k_var * MF_BINS1; i += BLOCK)
        partial[(size_t)blockIdx.x * k_var * MF_BINS1 + i] = h[i];
}

// One block per rank: totals, the check that makes the result exact, the round-1 bin.
__global__ __launch_bounds__(BLOCK) void ms_locate_kernel(MultiState* ms,
                                                          const uint32_t* __restrict__ cnt,
                                                          const uint32_t* __restrict__ partial,
                                                          uint32_t cap_sb) {
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t s_over;
    const uint32_t k = blockIdx.x, k_var = ms->k;
    const uint64_t p = ms->p[k];
    if (threadIdx.x == 0) s_over = 0;
    __syncthreads();
    static_assert(SPEC_SUB == BLOCK, "one split counter per thread");
    uint64_t below, inside;
    {
        uint32_t b = 0;
        for (uint32_t j = 0; j <= k; ++j) b += cnt[((size_t)(MC_BELOW + j) * SPEC_SUB + threadIdx.x) * 32u];
        block_excl_scan_u64(b, smem, &below);
        if (cnt[((size_t)MC_CAND * SPEC_SUB + threadIdx.x) * 32u] > cap_sb) s_over = 1;
    }
    // this rank's round-1 histogram: thread t owns bin t
    uint32_t c = 0;
#pragma unroll 8
    for (uint32_t q = 0; q < MF_BLOCKS; ++q)
        c += partial[((size_t)q * k_var + k) * MF_BINS1 + threadIdx.x];
    const uint64_t base = block_excl_scan_u64(c, smem, &inside);
    __syncthreads();
    if (s_over || !(below < p && p <= below + inside)) {
        if (threadIdx.x == 0) atomicOr(&ms->status, 1u);
        return;
    }
    const uint64_t r = p - below;
    if (base < r && r <= base + c) {
        ms->bin[k] = threadIdx.x;
        ms->bin_cnt[k] = c;
        ms->r2[k] = r - base;
        ms->less[k] = below + base;
        if (c > SPEC_LIST_CAP) atomicOr(&ms->status, 1u);
    }
}

// Candidates of each rank's selected bin -> that rank's list, one segment per block
// (LDS counters only: no global atomics).
__global__ __launch_bounds__(BLOCK) void ms_filter_kernel(MultiState* ms,
                                                          const uint32_t* __restrict__ cnt,
                                                          const uint2* __restrict__ cand,
                                                          uint32_t cap_sb, uint2* __restrict__ seg,
                                                          uint32_t* __restrict__ seg_cnt) {
    __shared__ uint32_t s_lo[MAXK + 1], s_hi[MAXK + 1], s_sh[MAXK], s_bin[MAXK], s_n[MAXK];
    const uint32_t k_var = ms->k;
    if (ms->status & 1u) return;
    if (threadIdx.x <= MAXK) {
        s_lo[threadIdx.x] = threadIdx.x < MAXK ? ms->lo[threadIdx.x] : 0xffffffffu;
        s_hi[threadIdx.x] = threadIdx.x < MAXK ? ms->hi[threadIdx.x] : 0xffffffffu;
        if (threadIdx.x < MAXK) {
            s_sh[threadIdx.x] = ms->sh[threadIdx.x];
            s_bin[threadIdx.x] = ms->bin[threadIdx.x];
            s_n[threadIdx.x] = 0;
        }
    }
    __syncthreads();
    ms_for_each_candidate(cnt, cand, cap_sb, [&](uint2 c, bool valid) {
        if (!valid) return;
        const uint32_t key = c.x & 0x7fffffffu;
        uint32_t ka, kb;
        rank_range(s_lo, s_hi, key, &ka, &kb);
        for (uint32_t k = ka; k < kb; ++k) {
            if (((key - s_lo[k]) >> s_sh[k]) == s_bin[k]) {
                const uint32_t pos = atomicAdd(&s_n[k], 1u);
                if (pos < SPEC_SEG_CAP)
                    seg[((size_t)k * MF_BLOCKS + blockIdx.x) * SPEC_SEG_CAP + pos] = c;
            }
        }
    });
    __syncthreads();
    if (threadIdx.x < k_var) {
        const uint32_t nn = s_n[threadIdx.x];
        seg_cnt[threadIdx.x * MF_BLOCKS + blockIdx.x] = min(nn, SPEC_SEG_CAP);
        if (nn > SPEC_SEG_CAP) atomicOr(&ms->status, 1u);
    }
}

// One block per rank: round-2 histogram over the rank's list (thread t walks segment t),
// exact rank by counting inside the selected bin, the record.
__global__ __launch_bounds__(BLOCK) void ms_rank_kernel(MultiState* ms,
                                                        const uint2* __restrict__ seg,
                                                        const uint32_t* __restrict__ seg_cnt,
                                                        shifter_threshold* thr) {
    __shared__ uint32_t h[MF_BINS2];
    __shared__ uint64_t comp[SPEC_SMALL_CAP];
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint64_t s_sel, s_less2, s_r3;
    __shared__ uint32_t s_lt, s_eq, s_bin2, s_cnt2, s_nb;
    const uint32_t k = blockIdx.x;
    shifter_threshold out;
    out.reserved = 0;
    out.n_prune = ms->p[k];
    shifter_threshold* dst = thr + ms->perm[k];
    if (ms->status & 1u) return;
    static_assert(MF_BLOCKS == BLOCK, "one list segment per thread");
    const uint32_t my_n = seg_cnt[k * MF_BLOCKS + threadIdx.x];
    const uint2* my_seg = seg + ((size_t)k * MF_BLOCKS + threadIdx.x) * SPEC_SEG_CAP;
    uint64_t n_tot;
    block_excl_scan_u64(my_n, smem, &n_tot);
    if (n_tot != ms->bin_cnt[k]) {   // cannot happen unless the buffers were disturbed
        if (threadIdx.x == 0) atomicOr(&ms->status, 1u);
        return;
    }
    const uint32_t sh = ms->sh[k];
    const uint32_t sh2 = sh > 12 ? sh - 12 : 0;   // 2^sh keys over 2^12 bins
    const uint32_t lo1 = ms->lo[k] + (ms->bin[k] << sh);
    for (uint32_t i = threadIdx.x; i < MF_BINS2; i += BLOCK) h[i] = 0;
    if (threadIdx.x == 0) { s_lt = 0; s_eq = 0; s_sel = 0; s_nb = 0; s_cnt2 = 0; s_bin2 = 0; }
    __syncthreads();
    for (uint32_t i = 0; i < my_n; ++i) atomicAdd(&h[((my_seg[i].x & 0x7fffffffu) - lo1) >> sh2], 1u);
    __syncthreads();
    constexpr uint32_t PER = MF_BINS2 / BLOCK;
    const uint32_t b0 = threadIdx.x * PER;
    uint64_t sum = 0, tot;
    for (uint32_t i = 0; i < PER; ++i) sum += h[b0 + i];
    uint64_t base = block_excl_scan_u64(sum, smem, &tot);
    const uint64_t r = ms->r2[k];
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
        if (threadIdx.x == 0) atomicOr(&ms->status, 1u);
        return;
    }
    for (uint32_t i = 0; i < my_n; ++i) {
        const uint2 c = my_seg[i];
        const uint32_t key = c.x & 0x7fffffffu;
        if (((key - lo1) >> sh2) == bin2) {
            const uint32_t pos = atomicAdd(&s_nb, 1u);
            comp[pos] = ((uint64_t)key << 32) | c.y;   // pos < cnt2 <= SPEC_SMALL_CAP
        }
    }
    __syncthreads();
    const uint64_t want = s_r3 - 1;
    for (uint32_t i = threadIdx.x; i < cnt2; i += BLOCK) {
        const uint64_t c = comp[i];
        uint32_t rank = 0;
        for (uint32_t f = 0; f < cnt2; ++f) rank += comp[f] < c;
        if (rank == want) s_sel = c;
    }
    __syncthreads();
    const uint64_t sel = s_sel;
    const uint32_t key = (uint32_t)(sel >> 32);
    uint32_t lt = 0, eq = 0;
    for (uint32_t i = threadIdx.x; i < cnt2; i += BLOCK) {
        const uint32_t kk = (uint32_t)(comp[i] >> 32);
        lt += kk < key;
        eq += kk == key;
    }
    if (lt) atomicAdd(&s_lt, lt);
    if (eq) atomicAdd(&s_eq, eq);
    __syncthreads();
    if (threadIdx.x == 0) {
        out.t_key = key;
        out.g_cut = sel & 0xffffffffull;
        out.cut = sel + 1;
        out.n_less = ms->less[k] + s_less2 + s_lt;
        out.n_equal = s_eq;
        *dst = out;
    }
}

void launch_spec_multi(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                       const PruneCounts& sorted_p, const MultiPerm& perm, uint32_t k,
                       uint64_t zero_mask, shifter_threshold* d_thr) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size();
    hipStream_t s = ctx->stream;
    {
        ProfileScope ps(ctx, K_SPEC_INIT);
        ms_init_kernel<<<64, BLOCK, 0, s>>>(b.multi, b.shist, b.multi_cnt, sorted_p, perm, k,
                                            m->sample_size, zero_mask, d_thr);
    }
    if (k == 0) return;   // every count was zero
    {
        ProfileScope ps(ctx, K_SPEC_SAMPLE);
        launch_spec_sample(ctx, m, d_w);
    }
    {
        ProfileScope ps(ctx, K_SPEC_PREDICT);
        ms_predict_kernel<<<1, BLOCK, 0, s>>>(b.multi, b.shist, m->info.n_prunable,
                                              ctx->margin_sigmas);
    }
    {
        ProfileScope ps(ctx, K_SPEC_PASS);
        const bool nt = m->info.w_extent * 4 > (192ull << 20);
        auto kern = nt ? ms_pass_kernel<true> : ms_pass_kernel<false>;
        kern<<<m->n_tiles, BLOCK, 0, s>>>(b.tens, b.tile_prefix, n_t, d_w, b.multi, b.multi_cnt,
                                          b.cand, b.cand_cap_sb);
    }
    {
        ProfileScope ps(ctx, K_SPEC_FINISH);
        ms_hist_kernel<<<MF_BLOCKS, BLOCK, k * MF_BINS1 * sizeof(uint32_t), s>>>(
            b.multi, b.multi_cnt, b.cand, b.cand_cap_sb, b.multi_partial);
        ms_locate_kernel<<<k, BLOCK, 0, s>>>(b.multi, b.multi_cnt, b.multi_partial, b.cand_cap_sb);
    }
    {
        ProfileScope ps(ctx, K_SPEC_FINISH2);
        ms_filter_kernel<<<MF_BLOCKS, BLOCK, 0, s>>>(b.multi, b.multi_cnt, b.cand, b.cand_cap_sb,
                                                     b.multi_seg, b.multi_seg_cnt);
        ms_rank_kernel<<<k, BLOCK, 0, s>>>(b.multi, b.multi_seg, b.multi_seg_cnt, d_thr);
    }
}

}  // namespace shifter
