// Single-pass exact selection for ALL prune counts of a portfolio at once: the ranking of
// Sec. II-A / Sec. III-C of the paper for K sparsity levels in one read of the arena.
//
// Same scheme as the one-count selection (sample, predict, one pass, finish), with the
// prune counts sorted ascending so that the predicted key intervals [lo_k, hi_k] have
// non-decreasing ends.  Intervals that overlap are merged into one (a cluster of ranks
// sharing lo and hi), so two intervals are either the same or disjoint.  For a weight with
// key x let j = #{k : lo_k <= x}; then
//   x < lo_k  <=>  j <= k            (so below_k is a prefix sum of the counts per j)
//   x is a candidate  <=>  j >= 1 and x <= hi_{j-1}; it belongs to the cluster whose last
//                          rank is j - 1
// so one search per weight replaces K interval tests.  The pass appends a candidate to the
// region of its cluster (split 256 ways by block, one reservation per block and cluster);
// the finish is one launch, one block per rank, which walks its cluster's region.
#include "dev_common.h"

namespace shifter {

constexpr uint32_t MS_BINS = SAMPLE_BINS;   // sample histogram bins (sample_bin)
constexpr uint32_t TAB_SHIFT = 19;       // the pass's bucket table: 4096 buckets of 2^19 keys
constexpr uint32_t TAB_SIZE = 1u << (31 - TAB_SHIFT);
// The counters all blocks add to are split CAND_SUB ways by block (one 128-byte line per
// part), and so is a cluster's candidate region: few enough parts that each averages over
// hundreds of tiles - filters differ in scale by orders of magnitude, so the candidates of
// one threshold crowd into few tiles - and enough that the additions of all blocks do not
// queue on one address.
constexpr uint32_t CAND_SUB = 32;
static_assert(CAND_SUB <= SPEC_SUB, "the counters use the first CAND_SUB lines of a row");
constexpr uint32_t FIN_THREADS = 1024;   // the last step of the finish: one block per rank
constexpr uint32_t FIN_BINS = 4096;      // bins of one refinement level there
constexpr uint32_t FIN_LIST = 1024;      // pairs the last bin may hold (too many equal keys beyond that)
constexpr uint32_t FIN_DIRECT = 96;      // pairs ranked by counting without refining further

// Split counters, one 128-byte line each: row j (0 <= j <= MAXK) counts the weights with
// exactly j lower ends at or below their key; row MAXK + 1 + r the candidates appended to
// the region of the cluster whose last rank is r.
__device__ __forceinline__ uint32_t* mcnt_below(uint32_t* cnt, uint32_t j, uint32_t sb) {
    return cnt + ((size_t)j * SPEC_SUB + sb) * 32u;
}
__device__ __forceinline__ uint32_t* mcnt_cand(uint32_t* cnt, uint32_t r, uint32_t sb) {
    return cnt + ((size_t)(MAXK + 1u + r) * SPEC_SUB + sb) * 32u;
}

// #{k : lo_k <= key} by a branch-free binary search; s_lo holds MAXK + 1 entries, padded
// with 0xffffffff.
__device__ __forceinline__ uint32_t count_lower_ends(const uint32_t* s_lo, uint32_t key) {
    uint32_t j = 0;
#pragma unroll
    for (uint32_t step = MAXK / 2; step >= 1; step >>= 1)
        if (s_lo[j + step - 1] <= key) j += step;
    return j + (s_lo[j] <= key ? 1u : 0u);
}

// One block.  First the set-up of a ranking (the state, the zero-count records; the sample
// histogram is read into registers and cleared for the next call), then the
// inclusive prefix of the sample histogram in LDS, for every rank the interval from the
// sample's order statistics at P/N -/+ margin, monotone ends, clusters, and each cluster's
// share of the candidate buffer.
// sorted_p / perm: the k prune counts > 0 in ascending order and their original positions;
// zero_mask: bit i set = original position i asked for P = 0 and gets its record here.
constexpr uint32_t PREDICT_THREADS = 1024;

__global__ __launch_bounds__(PREDICT_THREADS) void ms_predict_kernel(
    MultiState* ms, uint32_t* shist, uint32_t* cnt, PruneCounts sorted_p, MultiPerm perm,
    uint32_t k_var, uint32_t m, uint64_t zero_mask, shifter_threshold* thr,
    shifter_threshold* host_rec, uint64_t n_prunable, double margin_sigmas,
    uint8_t* __restrict__ tab, uint32_t cap_sb_total) {
    constexpr uint32_t SEG = 256, NSEG = MS_BINS / SEG, WAVES = PREDICT_THREADS / 64;
    static_assert(NSEG == 64, "one segment per lane in the scan of the segment sums");
    __shared__ uint32_t prefix[MS_BINS];          // 64 KB
    __shared__ uint32_t seg_sum[NSEG];
    __shared__ uint32_t s_total;
    __shared__ uint32_t s_lo[MAXK];
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    constexpr uint32_t PER_WAVE = NSEG / WAVES;   // segments per wavefront
    // each wavefront's segments are loaded once, all loads in flight together; the bins
    // are then cleared: the next ranking's sample adds to them
    uint4 x[PER_WAVE];
#pragma unroll
    for (uint32_t i = 0; i < PER_WAVE; ++i)
        x[i] = reinterpret_cast<const uint4*>(shist + (wid + i * WAVES) * SEG)[lane];
#pragma unroll
    for (uint32_t i = 0; i < PER_WAVE; ++i)
        reinterpret_cast<uint4*>(shist + (wid + i * WAVES) * SEG)[lane] = make_uint4(0, 0, 0, 0);
    if (threadIdx.x < MAXK) {
        const uint32_t t = threadIdx.x;
        ms->p[t] = t < k_var ? sorted_p.p[t] : 0;
        ms->perm[t] = t < k_var ? perm.v[t] : 0;
        if (t >= k_var) {                  // padding sorts last in the searches
            ms->lo[t] = 0xffffffffu;
            ms->hi[t] = 0xffffffffu;
            ms->mid[t] = 0xffffffffu;
            ms->clast[t] = t;
            ms->cand_off[t] = 0;
            ms->cand_cap[t] = 0;
        }
        if ((zero_mask >> t) & 1ull) {
            shifter_threshold out;
            out.cut = 0; out.t_key = 0; out.reserved = 0; out.g_cut = ~0ull; out.n_prune = 0;
            out.n_less = 0; out.n_equal = 0;
            thr[t] = out;
            host_rec[t] = out;
        }
    }
    if (threadIdx.x == 0) {
        ms->k = k_var;
        ms->m_valid = m;
        ms->status = 0;
    }
    if (k_var == 0) return;
    const uint64_t p = threadIdx.x < k_var ? sorted_p.p[threadIdx.x] : 0;
    // phase 1: segment sums, then their exclusive scan by the first wavefront
#pragma unroll
    for (uint32_t i = 0; i < PER_WAVE; ++i) {
        uint32_t v = x[i].x + x[i].y + x[i].z + x[i].w;
        for (uint32_t d = 32; d > 0; d >>= 1) v += __shfl_down(v, d, 64);
        if (lane == 0) seg_sum[wid + i * WAVES] = v;
    }
    __syncthreads();
    if (wid == 0) {
        const uint32_t v = seg_sum[lane];
        uint32_t incl = v;
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(incl, d, 64);
            if (lane >= d) incl += y;
        }
        seg_sum[lane] = incl - v;                 // exclusive segment base
        if (lane == 63) s_total = incl;
    }
    __syncthreads();
    const uint64_t total = s_total;
    // phase 2: inclusive prefix per bin
#pragma unroll
    for (uint32_t i = 0; i < PER_WAVE; ++i) {
        const uint32_t sg = wid + i * WAVES;
        const uint32_t mine4 = x[i].x + x[i].y + x[i].z + x[i].w;
        uint32_t incl = mine4;
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(incl, d, 64);
            if (lane >= d) incl += y;
        }
        uint32_t run = seg_sum[sg] + incl - mine4;
        uint32_t* out = prefix + sg * SEG + lane * 4;
        run += x[i].x; out[0] = run;
        run += x[i].y; out[1] = run;
        run += x[i].z; out[2] = run;
        run += x[i].w; out[3] = run;
    }
    __syncthreads();
    // the first wavefront: lane k takes rank k (k_var <= 64)
    if (wid == 0) {
        uint32_t lo = 0, hi = 0x7fffffffu, mid = 0;
        if (lane < k_var && p > 0 && m >= 256 && n_prunable > 0 && total == m) {
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
            if (r_lo > 0.0) lo = sample_bin_first_key(bin_of(r_lo));
            if (r_hi < (double)(m - 1)) hi = sample_bin_last_key(bin_of(r_hi));
            mid = sample_bin_first_key(bin_of(min(max(centre, 0.0), (double)(m - 1))));
        }
        // widen so that both ends are non-decreasing in k (ranks are sorted by P): a running
        // maximum of hi from the left, a running minimum of lo from the right; lanes past
        // the last rank hold the neutral values
        if (lane >= k_var) { lo = 0xffffffffu; hi = 0; }
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t yh = __shfl_up(hi, d, 64);
            const uint32_t yl = __shfl_down(lo, d, 64);
            if (lane >= d) hi = max(hi, yh);
            if (lane + d < 64) lo = min(lo, yl);
        }
        // clusters: rank k opens one unless its interval meets that of rank k - 1; every
        // rank of a cluster takes the first one's lo and the last one's hi
        const uint32_t hi_prev = __shfl_up(hi, 1, 64);
        const bool opens = lane < k_var && (lane == 0 || lo > hi_prev);
        const unsigned long long open_mask = __ballot(opens);
        const unsigned long long upto = open_mask & (~0ull >> (63u - lane));     // openers at or below this lane
        const uint32_t first = upto ? 63u - (uint32_t)__clzll(upto) : 0u;
        const unsigned long long after = lane < 63u ? open_mask >> (lane + 1u) : 0ull;   // openers above it
        uint32_t last = after ? lane + (uint32_t)__ffsll(after) - 1u : k_var - 1u;
        if (lane >= k_var) last = lane;
        lo = __shfl(lo, first, 64);
        hi = __shfl(hi, min(last, 63u), 64);
        // provisional threshold of the fused pass: inside the interval, non-decreasing (a
        // running maximum: it stays below hi because hi is non-decreasing)
        uint32_t pm = lane < k_var ? min(max(mid, lo), hi) : 0u;
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(pm, d, 64);
            if (lane >= d) pm = max(pm, y);
        }
        // each cluster's share of the candidate buffer, in proportion to the samples inside
        // its interval (plus a little for the empty ones); the region belongs to the
        // cluster's last rank
        uint32_t wt = 0;
        if (lane < k_var && last == lane) {
            const uint32_t b_lo = sample_bin(lo), b_hi = sample_bin(hi);
            wt = prefix[b_hi] - (b_lo ? prefix[b_lo - 1u] : 0u) + 64u;
        }
        uint64_t wsum = wt;
        for (uint32_t d = 32; d > 0; d >>= 1) wsum += __shfl_down(wsum, d, 64);
        wsum = __shfl(wsum, 0, 64);
        // cap_sb_total pairs per 1/SPEC_SUB of the buffer; a part of a region is 1/CAND_SUB of it
        const uint32_t cap = wt ? (uint32_t)((uint64_t)cap_sb_total * (SPEC_SUB / CAND_SUB) * wt / wsum) : 0u;
        uint32_t cinc = cap;
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t y = __shfl_up(cinc, d, 64);
            if (lane >= d) cinc += y;
        }
        if (lane < k_var) {
            ms->lo[lane] = lo;
            ms->hi[lane] = hi;
            ms->mid[lane] = pm;
            ms->clast[lane] = last;
            ms->cand_cap[lane] = cap;
            ms->cand_off[lane] = (cinc - cap) * CAND_SUB;     // at most cap_sb_total * SPEC_SUB pairs
            s_lo[lane] = lo;
        }
        // the finish's view of a rank: its cluster's region and first histogram
        const uint32_t cap_cl = __shfl(cap, min(last, 63u), 64);
        const uint32_t off_cl = __shfl((cinc - cap) * CAND_SUB, min(last, 63u), 64);
        if (lane < k_var) {
            const uint32_t span = hi - lo;
            RankIn in;
            in.p = p;
            in.lo = lo;
            in.sh = span < 256u ? 0u : (32u - (uint32_t)__clz(span)) - 8u;
            in.clast = last;
            in.cand_off = off_cl;
            in.cand_cap = cap_cl;
            in.perm = perm.v[lane];
            ms->rin[lane] = in;
        }
    }
    // The pass's bucket table.  Entry b covers the keys [b << TAB_SHIFT, (b + 1) << TAB_SHIFT):
    // bits 0-5 = #{k : lo_k <= first key of the bucket}, bits 6-7 = how many lo_k lie
    // above that inside the bucket (3: three or more).  With a few dozen ranks almost every
    // bucket holds none, and a weight's j is then the entry itself.
    __syncthreads();
    constexpr uint32_t PER_THREAD = TAB_SIZE / PREDICT_THREADS;
    uint32_t j0[PER_THREAD], inside[PER_THREAD];
#pragma unroll
    for (uint32_t i = 0; i < PER_THREAD; ++i) j0[i] = inside[i] = 0;
    for (uint32_t k = 0; k < k_var; ++k) {
        const uint32_t lo = s_lo[k];
#pragma unroll
        for (uint32_t i = 0; i < PER_THREAD; ++i) {
            const uint32_t first = (threadIdx.x + i * PREDICT_THREADS) << TAB_SHIFT;
            const uint32_t last = first + ((1u << TAB_SHIFT) - 1u);
            j0[i] += lo <= first ? 1u : 0u;
            inside[i] += (lo > first && lo <= last) ? 1u : 0u;
        }
    }
#pragma unroll
    for (uint32_t i = 0; i < PER_THREAD; ++i)
        tab[threadIdx.x + i * PREDICT_THREADS] = (uint8_t)(j0[i] | (min(inside[i], 3u) << 6));
}

// Appends the candidates a block found to the regions of their clusters: count per cluster
// in LDS, one global reservation per cluster the block met, then the writes.  `for_each`
// calls its argument once per candidate of the calling thread with (bits, global index,
// cluster = last rank whose lower end lies at or below the key).  All threads of the block
// call this; it contains barriers.
template <typename ForEach>
__device__ __forceinline__ void ms_append_candidates(
    bool have, const uint32_t* s_coff, const uint32_t* s_ccap, uint32_t* s_rc, uint32_t* s_rc2,
    uint32_t* s_rbase, uint32_t k_var, uint32_t* cnt, uint32_t csb, uint2* __restrict__ cand,
    ForEach&& for_each) {
    if (!__syncthreads_or(have ? 1 : 0)) return;      // uniform: no candidate in this block
    if (have) for_each([&](uint32_t, uint32_t, uint32_t cl) { atomicAdd(&s_rc[cl], 1u); });
    __syncthreads();
    if (threadIdx.x < k_var) {
        const uint32_t c = s_rc[threadIdx.x];
        if (c) s_rbase[threadIdx.x] = atomicAdd(mcnt_cand(cnt, threadIdx.x, csb), c);
    }
    __syncthreads();
    if (have)
        for_each([&](uint32_t bits, uint32_t g, uint32_t cl) {
            const uint32_t pos = s_rbase[cl] + atomicAdd(&s_rc2[cl], 1u);
            const uint32_t cap = s_ccap[cl];
            if (pos < cap) cand[(size_t)s_coff[cl] + (size_t)csb * cap + pos] = make_uint2(bits, g);
        });
}

// The one pass over the arena: counts per j and candidate pairs.
template <bool NT>
__global__ __launch_bounds__(BLOCK) void ms_pass_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix, uint32_t n_t,
    const float* __restrict__ w, MultiState* ms, uint32_t* cnt, uint2* __restrict__ cand,
    const uint8_t* __restrict__ tab, uint32_t* zero_ptr, uint32_t zero_n) {
    // an array the step behind this pass wants cleared (or nullptr)
    for (uint32_t i = blockIdx.x * BLOCK + threadIdx.x; i < zero_n; i += gridDim.x * BLOCK) zero_ptr[i] = 0;
    // s_hi1[j] = hi_(j-1) + 1, s_hi1[0] = 0: a weight with j lower ends at or below it is a
    // candidate (of the cluster ending at rank j - 1) iff key < s_hi1[j]
    __shared__ uint32_t s_lo[MAXK + 1], s_hi1[MAXK + 1];
    __shared__ uint32_t s_coff[MAXK], s_ccap[MAXK], s_rc[MAXK], s_rc2[MAXK], s_rbase[MAXK];
    // counts per j: one private byte column per thread (a thread sees 16 weights; no
    // conflicts, no atomics), summed at the end; rows 0 .. k_var of BLOCK bytes (the launch
    // sizes it).  Small, so that a CU holds as many blocks as it has wavefront slots: a
    // block's life is a chain of memory latencies, which only other blocks can hide.
    extern __shared__ uint32_t s_col[];
    __shared__ __align__(16) uint8_t s_tab[TAB_SIZE];
    __shared__ uint32_t s_nan;
    const uint32_t tile = blockIdx.x;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    if (!tens[t].prunable) return;
    const DevTensor T = tens[t];
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const uint32_t g0 = (uint32_t)(T.gbase + e0);
    const uint32_t sb = blockIdx.x & (SPEC_SUB - 1);
    // the tile's loads go out first: the set-up below runs while they are in flight
    const float* src = w + T.offset + e0;
    const bool whole = n == TILE && (T.offset & 3u) == 0;
    constexpr uint32_t U = TILE / BLOCK / 4;
    uint4 v[U];
    if (whole) {
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) v[u] = load_u4<NT>(s4 + threadIdx.x + BLOCK * u);
    }
    const uint32_t k_var = ms->k;
    if (threadIdx.x <= MAXK) {
        s_lo[threadIdx.x] = threadIdx.x < MAXK ? ms->lo[threadIdx.x] : 0xffffffffu;
        s_hi1[threadIdx.x] = (threadIdx.x >= 1 && threadIdx.x <= k_var) ? ms->hi[threadIdx.x - 1] + 1u : 0u;
    }
    if (threadIdx.x < MAXK) {
        s_coff[threadIdx.x] = ms->cand_off[threadIdx.x];
        s_ccap[threadIdx.x] = ms->cand_cap[threadIdx.x];
        s_rc[threadIdx.x] = 0;
        s_rc2[threadIdx.x] = 0;
    }
    for (uint32_t i = threadIdx.x; i < (k_var + 1) * (BLOCK / 4); i += BLOCK) s_col[i] = 0;
    static_assert(TAB_SIZE == BLOCK * 16, "one 16-byte piece of the table per thread");
    reinterpret_cast<uint4*>(s_tab)[threadIdx.x] = reinterpret_cast<const uint4*>(tab)[threadIdx.x];
    if (threadIdx.x == 0) s_nan = 0;
    __syncthreads();

    uint32_t key_max = 0;   // a NaN's key is above that of +inf
    uint8_t* my_col = reinterpret_cast<uint8_t*>(s_col) + threadIdx.x;
    // classify one weight; returns whether it is a candidate; adds it to the count of
    // j = #{k : lo_k <= key}: the bucket table's entry, plus a compare or two in the few
    // buckets that hold a rank's lower end (the binary search where three or more meet)
    auto one = [&](uint32_t bits, uint32_t& j_out) -> bool {
        const uint32_t key = bits & 0x7fffffffu;
        key_max = max(key_max, key);
        const uint32_t e = s_tab[key >> TAB_SHIFT];
        uint32_t j = e & 63u;
        if (e >> 6) {
            if ((e >> 6) == 3u) {
                j = count_lower_ends(s_lo, key);    // j in [0, MAXK]; s_lo[MAXK] is padding
            } else {
                // the lower ends are sorted: the second one counts only if the first does
                const uint32_t j0 = j;
                j += s_lo[j0] <= key ? 1u : 0u;
                j += ((e >> 6) == 2u && s_lo[j0 + 1] <= key) ? 1u : 0u;
            }
        }
        my_col[j * BLOCK] += 1;                 // private byte, at most 16
        j_out = j;
        return key < s_hi1[j];                  // j <= k_var <= SPEC_MULTI_MAXK
    };

    if (whole) {
        uint32_t cmask = 0, jj[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            uint32_t j_0, j_1, j_2, j_3;
            cmask |= ((one(v[u].x, j_0) ? 1u : 0u) | (one(v[u].y, j_1) ? 2u : 0u) |
                      (one(v[u].z, j_2) ? 4u : 0u) | (one(v[u].w, j_3) ? 8u : 0u)) << (4 * u);
            jj[u] = j_0 | (j_1 << 8) | (j_2 << 16) | (j_3 << 24);
        }
        ms_append_candidates(cmask != 0, s_coff, s_ccap, s_rc, s_rc2, s_rbase, k_var, cnt,
                             blockIdx.x & (CAND_SUB - 1), cand,
                             [&](auto&& f) {
#pragma unroll
                                 for (uint32_t u = 0; u < U; ++u) {
                                     const uint32_t j = (threadIdx.x + BLOCK * u) * 4;
                                     const uint32_t vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                                     for (uint32_t q = 0; q < 4; ++q)
                                         if (cmask & (1u << (4 * u + q)))
                                             f(vv[q], g0 + j + q, ((jj[u] >> (8 * q)) & 0xffu) - 1u);
                                 }
                             });
    } else {
        // ragged or unaligned tile (a few per tensor): one global atomic per candidate
        for (uint32_t j0 = 0; j0 < n; j0 += BLOCK) {
            const uint32_t j = j0 + threadIdx.x;
            if (j < n) {
                const uint32_t bits = __float_as_uint(src[j]);
                uint32_t jw;
                if (one(bits, jw)) {
                    const uint32_t cl = jw - 1u;
                    const uint32_t csb = blockIdx.x & (CAND_SUB - 1);
                    const uint32_t pos = atomicAdd(mcnt_cand(cnt, cl, csb), 1u);
                    const uint32_t cap = s_ccap[cl];
                    if (pos < cap) cand[(size_t)s_coff[cl] + (size_t)csb * cap + pos] = make_uint2(bits, g0 + j);
                }
            }
        }
    }
    if (key_max > 0x7f800000u) s_nan = 1;
    __syncthreads();
    // column sums: four threads per j, a quarter of the row's words each (rotated by j: the
    // rows start in the same bank); bytes are added in two 16-bit lanes per word
    if (threadIdx.x < 4 * (k_var + 1)) {
        const uint32_t j = threadIdx.x >> 2, q = threadIdx.x & 3u;
        constexpr uint32_t ROW_W = BLOCK / 4;
        uint32_t even = 0, odd = 0;
        for (uint32_t i = 0; i < ROW_W / 4; ++i) {
            const uint32_t x = s_col[j * ROW_W + ((q * (ROW_W / 4) + i + j) & (ROW_W - 1))];
            even += x & 0x00ff00ffu;
            odd += (x >> 8) & 0x00ff00ffu;
        }
        const uint32_t c = (even & 0xffffu) + (even >> 16) + (odd & 0xffffu) + (odd >> 16);
        if (c) atomicAdd(mcnt_below(cnt, j, sb), c);
    }
    if (threadIdx.x == 0 && s_nan) atomicOr(&ms->status, 2u);
}

// The finish, three launches over the candidates.
//   hist    grid (part, rank): a 256-bin histogram of (key - lo) >> sh over one part of a
//           cluster's region, added to the cluster's histogram in global memory;
//   filter  grid (part, rank): every block first locates its rank - totals of the split
//           counters, the check that makes the result exact (below < P <= below + candidates
//           of the cluster), the bin holding the P-th pair - and then moves its part's pairs
//           of that bin to the rank's list (one reservation per block);
//   rank    one block per rank: refines the list with 4096-bin histograms until a bin holds
//           at most FIN_LIST pairs, ranks those exactly by counting and writes the record,
//           to d_thr and to its mirror in pinned host memory, with the rank's status word
//           (bit 0: could not decide; bit 1: NaN; bit 2: a buffer was full or too many
//           weights share the threshold's key - wider intervals would not help).
constexpr uint32_t MF_THREADS = 1024, MF_DEPTH = 8;
constexpr uint32_t MF_BINS1 = 256;
constexpr uint32_t MF_STAGE = 2048;      // pairs of the selected bin one filter block may hold

// f(pair) for the n pairs at src, MF_DEPTH loads per thread in flight.
template <typename F>
__device__ __forceinline__ void ms_walk(const uint2* __restrict__ src, uint32_t n, F&& f) {
    for (uint32_t i0 = 0; i0 < n; i0 += MF_THREADS * MF_DEPTH) {
        uint2 c[MF_DEPTH];
#pragma unroll
        for (uint32_t u = 0; u < MF_DEPTH; ++u) {
            const uint32_t i = i0 + u * MF_THREADS + threadIdx.x;
            c[u] = i < n ? src[i] : make_uint2(0xffffffffu, 0xffffffffu);
        }
#pragma unroll
        for (uint32_t u = 0; u < MF_DEPTH; ++u)
            if (i0 + u * MF_THREADS + threadIdx.x < n) f(c[u]);
    }
}

__global__ __launch_bounds__(MF_THREADS) void ms_hist_kernel(
    const MultiState* __restrict__ ms, const uint32_t* __restrict__ cnt,
    const uint2* __restrict__ cand, uint32_t* ghist, uint64_t* rowsum, uint32_t k_var) {
    __shared__ uint32_t h[MF_BINS1];
    if (blockIdx.y == k_var) {
        // the layer of blocks past the ranks adds up the rows of split counters (row j:
        // weights with exactly j lower ends at or below their key), one row per wavefront
        static_assert(SPEC_SUB == 256, "four counters per lane");
        const uint32_t lane = threadIdx.x & 63u;
        const uint32_t j = blockIdx.x * (MF_THREADS / 64) + (threadIdx.x >> 6);
        if (j <= k_var) {
            uint64_t v = 0;
#pragma unroll
            for (uint32_t q = 0; q < SPEC_SUB / 64; ++q) v += cnt[((size_t)j * SPEC_SUB + q * 64u + lane) * 32u];
            for (uint32_t d = 32; d > 0; d >>= 1) v += __shfl_down(v, d, 64);
            if (lane == 0) rowsum[j] = v;
        }
        return;
    }
    const uint32_t part = blockIdx.x, cl = blockIdx.y;
    const RankIn R = ms->rin[cl];
    if (R.clast != cl) return;                       // only a cluster's last rank owns a region
    const uint32_t cap = R.cand_cap;
    const uint32_t n = min(cnt[((size_t)(MAXK + 1u + cl) * SPEC_SUB + part) * 32u], cap);
    if (n == 0) return;
    if (threadIdx.x < MF_BINS1) h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t lo = R.lo, sh = R.sh;
    ms_walk(cand + (size_t)R.cand_off + (size_t)part * cap, n,
            [&](uint2 c) { atomicAdd(&h[((c.x & 0x7fffffffu) - lo) >> sh], 1u); });
    __syncthreads();
    if (threadIdx.x < MF_BINS1) {
        const uint32_t c = h[threadIdx.x];
        if (c) atomicAdd(&ghist[cl * MF_BINS1 + threadIdx.x], c);
    }
}

__global__ __launch_bounds__(MF_THREADS) void ms_filter_kernel(
    MultiState* ms, const uint32_t* __restrict__ cnt, const uint2* __restrict__ cand,
    const uint32_t* __restrict__ ghist, const uint64_t* __restrict__ rowsum, uint2* __restrict__ list,
    uint32_t* list_cnt) {
    __shared__ uint64_t smem[MF_THREADS / 64 + 1];
    __shared__ uint2 stage[MF_STAGE];
    __shared__ uint32_t s_over, s_bin, s_found, s_n, s_base;
    const uint32_t part = blockIdx.x, k = blockIdx.y;
    const RankIn R = ms->rin[k];
    const uint32_t cl = R.clast;
    const uint64_t p = R.p;
    const uint32_t cap = R.cand_cap;
    const bool publish = part == 0;
    if (threadIdx.x == 0) { s_over = 0; s_found = 0; s_n = 0; s_bin = 0; }
    __syncthreads();
    // weights below the cluster's interval: rows 0 .. k of the split counters
    uint64_t below, inside;
    {
        const uint64_t b = threadIdx.x <= k ? rowsum[threadIdx.x] : 0;     // k < MAXK <= MF_THREADS
        uint32_t c = 0;
        if (threadIdx.x < CAND_SUB) {
            c = cnt[((size_t)(MAXK + 1u + cl) * SPEC_SUB + threadIdx.x) * 32u];
            if (c > cap) s_over = 1;
        }
        block_excl_scan_u64<MF_THREADS>(b, smem, &below);
        block_excl_scan_u64<MF_THREADS>(c, smem, &inside);
    }
    __syncthreads();
    uint32_t why = 0;
    if (s_over) why = 5u;
    else if (!(below < p && p <= below + inside)) why = 1u;
    uint64_t r = 0, base = 0;
    uint32_t c = 0;
    if (!why) {
        r = p - below;
        c = threadIdx.x < MF_BINS1 ? ghist[cl * MF_BINS1 + threadIdx.x] : 0u;
        uint64_t tot;
        base = block_excl_scan_u64<MF_THREADS>(c, smem, &tot);
        if (threadIdx.x < MF_BINS1 && base < r && r <= base + c) {
            s_bin = threadIdx.x;
            s_found = 1;
            if (publish) {
                RankOut* o = &ms->rout[k];
                o->bin = threadIdx.x;
                o->bin_cnt = c;
                o->r2 = r - base;
                o->less = below + base;
                if (c > SPEC_LIST_CAP) atomicOr(&o->fail, 5u);
            }
        }
        __syncthreads();
        if (!s_found) why = 1u;       // cannot happen unless the buffers were disturbed
    }
    if (why) {
        if (publish && threadIdx.x == 0) atomicOr(&ms->rout[k].fail, why);
        return;
    }
    // this part's pairs of the selected bin -> the rank's list
    const uint32_t n = min(cnt[((size_t)(MAXK + 1u + cl) * SPEC_SUB + part) * 32u], cap);
    const uint32_t lo = R.lo, sh = R.sh, bin = s_bin;
    ms_walk(cand + (size_t)R.cand_off + (size_t)part * cap, n, [&](uint2 x) {
        if ((((x.x & 0x7fffffffu) - lo) >> sh) == bin) {
            const uint32_t pos = atomicAdd(&s_n, 1u);
            if (pos < MF_STAGE) stage[pos] = x;
        }
    });
    __syncthreads();
    const uint32_t m = s_n;
    if (m > MF_STAGE) {
        if (threadIdx.x == 0) atomicOr(&ms->rout[k].fail, 5u);
        return;
    }
    if (m == 0) return;
    if (threadIdx.x == 0) s_base = atomicAdd(&list_cnt[k], m);
    __syncthreads();
    uint2* dst = list + (size_t)k * SPEC_LIST_CAP;
    for (uint32_t i = threadIdx.x; i < m; i += MF_THREADS)
        if (s_base + i < SPEC_LIST_CAP) dst[s_base + i] = stage[i];
}

__global__ __launch_bounds__(FIN_THREADS) void ms_rank_kernel(
    MultiState* ms, const uint2* __restrict__ list, const uint32_t* __restrict__ list_cnt,
    shifter_threshold* thr, shifter_threshold* host_rec, uint32_t* host_status) {
    __shared__ uint32_t h[FIN_BINS];
    __shared__ uint64_t comp[FIN_LIST];
    __shared__ uint64_t smem[FIN_THREADS / 64 + 1];
    __shared__ uint64_t s_sel, s_base;
    __shared__ uint32_t s_bin, s_cnt, s_lt, s_eq, s_nb;
    const uint32_t k = blockIdx.x;
    // everything this block needs from the state, fetched side by side
    const RankIn R = ms->rin[k];
    const RankOut O = ms->rout[k];
    const uint32_t n = list_cnt[k];
    const uint32_t nan_bit = ms->status & 2u;      // the pass has ended
    const uint64_t p = R.p;
    auto give_up = [&](uint32_t why) {
        if (threadIdx.x == 0) {
            atomicOr(&ms->status, 1u);
            host_status[k] = why | 1u | nan_bit;
        }
    };
    if (O.fail) { give_up(O.fail); return; }
    if (n != O.bin_cnt || n > SPEC_LIST_CAP) { give_up(5u); return; }
    const uint2* src = list + (size_t)k * SPEC_LIST_CAP;
    if (threadIdx.x == 0) { s_sel = 0; s_nb = 0; s_lt = 0; s_eq = 0; }
    uint64_t r = O.r2;               // 1-based rank among the pairs still in play
    uint64_t less = O.less;          // weights below them
    uint32_t width_sh = R.sh;        // the pairs in play have (key - lo_cur) >> width_sh == 0
    uint32_t lo_cur = R.lo + (O.bin << width_sh);
    uint32_t cnt_sel = n;
    // refine while it pays: ranking by counting is quadratic; a bin of equal keys cannot be
    // refined and must fit the list
    while (cnt_sel > FIN_DIRECT) {
        if (width_sh == 0) {
            if (cnt_sel > FIN_LIST) { give_up(5u); return; }   // the multi-pass select ranks so many ties
            break;
        }
        const uint32_t sh = width_sh > 12u ? width_sh - 12u : 0u;
        for (uint32_t i = threadIdx.x; i < FIN_BINS; i += FIN_THREADS) h[i] = 0;
        __syncthreads();
        ms_walk(src, n, [&](uint2 c) {
            const uint32_t d = (c.x & 0x7fffffffu) - lo_cur;      // wraps for keys below lo_cur
            if ((d >> width_sh) == 0) atomicAdd(&h[d >> sh], 1u);
        });
        __syncthreads();
        constexpr uint32_t PER = FIN_BINS / FIN_THREADS;
        const uint32_t b0 = threadIdx.x * PER;
        uint64_t sum = 0, tot;
        uint32_t c4[PER];
#pragma unroll
        for (uint32_t i = 0; i < PER; ++i) { c4[i] = h[b0 + i]; sum += c4[i]; }
        uint64_t base = block_excl_scan_u64<FIN_THREADS>(sum, smem, &tot);
        if (base < r && r <= base + sum) {
#pragma unroll
            for (uint32_t i = 0; i < PER; ++i) {
                if (base < r && r <= base + c4[i]) { s_bin = b0 + i; s_cnt = c4[i]; s_base = base; }
                base += c4[i];
            }
        }
        __syncthreads();
        if (tot < r) { give_up(1u); return; }    // cannot happen unless the buffers were disturbed
        less += s_base;
        r -= s_base;
        lo_cur += s_bin << sh;
        width_sh = sh;
        cnt_sel = s_cnt;
        __syncthreads();
    }
    __syncthreads();
    // the pairs of the last bin, then the r-th of them by counting
    ms_walk(src, n, [&](uint2 c) {
        const uint32_t key = c.x & 0x7fffffffu, d = key - lo_cur;
        if ((d >> width_sh) == 0) {
            const uint32_t pos = atomicAdd(&s_nb, 1u);
            if (pos < FIN_LIST) comp[pos] = ((uint64_t)key << 32) | c.y;
        }
    });
    __syncthreads();
    if (s_nb != cnt_sel || r == 0 || r > cnt_sel) { give_up(1u); return; }
    const uint64_t want = r - 1;
    for (uint32_t i = threadIdx.x; i < cnt_sel; i += FIN_THREADS) {
        const uint64_t c = comp[i];
        uint32_t rank = 0;
        for (uint32_t f = 0; f < cnt_sel; ++f) rank += comp[f] < c;
        if (rank == want) s_sel = c;        // composites are distinct: exactly one hit
    }
    __syncthreads();
    const uint64_t sel = s_sel;
    const uint32_t key = (uint32_t)(sel >> 32);
    uint32_t lt = 0, eq = 0;
    for (uint32_t i = threadIdx.x; i < cnt_sel; i += FIN_THREADS) {
        const uint32_t kk = (uint32_t)(comp[i] >> 32);
        lt += kk < key;
        eq += kk == key;
    }
    if (lt) atomicAdd(&s_lt, lt);
    if (eq) atomicAdd(&s_eq, eq);
    __syncthreads();
    if (threadIdx.x == 0) {
        shifter_threshold out;
        out.reserved = 0;
        out.n_prune = p;
        out.t_key = key;
        out.g_cut = sel & 0xffffffffull;
        out.cut = sel + 1;
        out.n_less = less + s_lt;
        out.n_equal = s_eq;
        thr[R.perm] = out;
        host_rec[R.perm] = out;
        host_status[k] = nan_bit;
    }
}

// ---------------------------------------------------------------------------------------
// Steps 1-3 for the K variants of a portfolio in ONE read of the arena: ms_pass_kernel's
// counting and candidate capture merged with the batched mask pass.  For a weight with
// j = #{r : lo_r <= key} over the sorted ranks, rank r removes it for sure when r >= j and
// keeps it for sure when hi_r < key; in between it is a candidate of r.  The pass writes
// every variant's sparse weight and mask byte - candidates provisionally - and the
// levels of the weights that are no rank's candidate; ms_fixup_kernel, once the exact cuts
// are known, rewrites the candidates written on the wrong side of their rank's cut (the
// pass decides by the predicted threshold mid of the last rank) and adds their levels.
// rv[v] = sorted rank of variant v, or -1 for a variant that removes nothing (P = 0).
struct VariantRanks {
    int32_t r[MAXK];
};

typedef uint32_t ms_uint4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // dword-aligned

template <bool NT>
__global__ __launch_bounds__(BLOCK) void ms_fused_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix, uint32_t n_t,
    const float* __restrict__ w, MultiState* ms, uint32_t* cnt, uint2* __restrict__ cand,
    VariantRanks rv, uint32_t k_all, float* __restrict__ w_out,
    uint64_t w_stride, uint8_t* __restrict__ mask, uint64_t mask_stride, uint32_t* out_level,
    uint32_t* in_level) {
    __shared__ uint32_t rowmax[TILE + 16];
    __shared__ uint32_t colmax[TILE + 16];
    __shared__ uint32_t s_lo[MAXK + 1], s_hi[MAXK + 1], s_mid[MAXK + 1];
    __shared__ uint32_t s_coff[MAXK], s_ccap[MAXK], s_rc[MAXK], s_rc2[MAXK], s_rbase[MAXK];
    __shared__ int32_t s_rv[MAXK];
    __shared__ uint8_t s_col[(SPEC_MULTI_MAXK + 1) * BLOCK];   // private counters, <= 16 each
    __shared__ __align__(16) uint32_t s_xm[TILE / 4];
    __shared__ uint32_t s_nan;

    const uint32_t tile = blockIdx.x;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    const DevTensor T = tens[t];
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const bool ranked = T.prunable != 0;
    const uint32_t g0 = (uint32_t)(T.gbase + e0);
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    const uint32_t sb = blockIdx.x & (SPEC_SUB - 1);
    const uint32_t k_var = ms->k;
    const uint32_t c0 = e0 % T.khw, r0 = e0 % T.row_len;
    const uint32_t nrows = (r0 + n - 1) / T.row_len + 1;
    const uint32_t ncols = (c0 + n - 1) / T.khw + 1;
    for (uint32_t s = threadIdx.x; s < nrows; s += BLOCK) rowmax[s] = 0;
    for (uint32_t s = threadIdx.x; s < ncols; s += BLOCK) colmax[s] = 0;
    if (threadIdx.x <= MAXK) {
        s_lo[threadIdx.x] = threadIdx.x < MAXK ? ms->lo[threadIdx.x] : 0xffffffffu;
        s_hi[threadIdx.x] = threadIdx.x < MAXK ? ms->hi[threadIdx.x] : 0xffffffffu;
        s_mid[threadIdx.x] = threadIdx.x < MAXK ? ms->mid[threadIdx.x] : 0xffffffffu;
    }
    if (threadIdx.x < MAXK) {
        s_rv[threadIdx.x] = rv.r[threadIdx.x];
        s_coff[threadIdx.x] = ms->cand_off[threadIdx.x];
        s_ccap[threadIdx.x] = ms->cand_cap[threadIdx.x];
        s_rc[threadIdx.x] = 0;
        s_rc2[threadIdx.x] = 0;
    }
    for (uint32_t j = 0; j <= k_var; ++j) s_col[j * BLOCK + threadIdx.x] = 0;
    if (threadIdx.x == 0) s_nan = 0;
    __syncthreads();

    uint32_t nan = 0;
    // number of ranks that keep one weight in what the pass writes (127 in tensors that are
    // not ranked: no rank removes it) and whether it is a candidate; counts it under
    // j = #{r : lo_r <= key}.  Ranks below j keep a weight that is no candidate.
    auto classify = [&](uint32_t bits, bool& is_cand, bool& below_mid) -> uint32_t {
        is_cand = false;
        below_mid = false;
        if (!ranked) return 127u;
        const uint32_t key = bits & 0x7fffffffu;
        nan |= key > 0x7f800000u ? 1u : 0u;
        uint32_t j = count_lower_ends(s_lo, key);
        is_cand = j >= 1 && key <= s_hi[j - 1];
        s_col[j * BLOCK + threadIdx.x] += 1;
        // a candidate is written as kept by the ranks below j - 1 and by rank j - 1 iff it
        // does not lie below that rank's predicted threshold (the fix-up settles it, in every
        // rank of its cluster)
        below_mid = is_cand && key < s_mid[j - 1];
        if (below_mid) j -= 1;
        return j;
    };
    auto mark = [&](uint32_t j, uint32_t bits, uint32_t level) {
        if (level && (bits & 0x7fffffffu)) {
            atomicMax(&rowmax[div_small(r0 + j, T.row_len, T.magic_row)], level);
            atomicMax(&colmax[div_small(c0 + j, T.khw, T.magic_khw)], level);
        }
    };

    const float* src = w + T.offset + e0;
    const bool want_mask = ranked && mask != nullptr;
    const bool vec_ok = n == TILE && (T.offset & 3u) == 0 && (!w_out || (w_stride & 3u) == 0) &&
                        (!want_mask || ((T.gbase & 3u) == 0 && (mask_stride & 3u) == 0));
    if (vec_ok) {
        constexpr uint32_t U = TILE / BLOCK / 4;
        const uint32_t q0 = wid * (64u * U) + lane;      // quad of step 0 (see the batched mask pass)
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
        uint4 v[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) v[u] = load_u4<NT>(s4 + q0 + 64u * u);
        uint32_t jj[U], cmask = 0, bmask = 0, lvl[U][4];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            bool c_0, c_1, c_2, c_3, b_0, b_1, b_2, b_3;
            const uint32_t j_0 = classify(v[u].x, c_0, b_0), j_1 = classify(v[u].y, c_1, b_1);
            const uint32_t j_2 = classify(v[u].z, c_2, b_2), j_3 = classify(v[u].w, c_3, b_3);
            jj[u] = j_0 | (j_1 << 8) | (j_2 << 16) | (j_3 << 24);
            cmask |= ((c_0 ? 1u : 0u) | (c_1 ? 2u : 0u) | (c_2 ? 4u : 0u) | (c_3 ? 8u : 0u)) << (4 * u);
            bmask |= ((b_0 ? 1u : 0u) | (b_1 ? 2u : 0u) | (b_2 ? 4u : 0u) | (b_3 ? 8u : 0u)) << (4 * u);
            lvl[u][0] = lvl[u][1] = lvl[u][2] = lvl[u][3] = 0;
        }
        uint32_t* xm = s_xm + wid * (64u * U);
        for (uint32_t k = 0; k < k_all; ++k) {
            const int32_t r = s_rv[k];
            float* dst = w_out + (uint64_t)k * w_stride + T.offset + e0;
            uint8_t* mdst = want_mask ? mask + (uint64_t)k * mask_stride + T.gbase + e0 : nullptr;
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t b[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
                uint32_t o[4], keep[4];
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    keep[q] = r < (int32_t)((jj[u] >> (8 * q)) & 0xffu) ? 1u : 0u;
                    o[q] = keep[q] ? b[q] : 0u;
                    lvl[u][q] += keep[q];
                }
                if (w_out)
                    store_u4<NT>(reinterpret_cast<uint4*>(dst) + q0 + 64u * u,
                                 make_uint4(o[0], o[1], o[2], o[3]));
                if (mdst) xm[64u * u + lane] = keep[0] | (keep[1] << 8) | (keep[2] << 16) | (keep[3] << 24);
            }
            if (mdst) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const uint4 mm = *reinterpret_cast<const uint4*>(xm + 4u * lane);
                ms_uint4_a4 out;
                out.x = mm.x; out.y = mm.y; out.z = mm.z; out.w = mm.w;
                *reinterpret_cast<ms_uint4_a4*>(mdst + wid * (256u * U) + 16u * lane) = out;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = (q0 + 64u * u) * 4;
            const uint32_t b[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q)
                if (!(cmask & (1u << (4 * u + q)))) mark(j + q, b[q], lvl[u][q]);
        }
        // candidate pairs: to the regions of their clusters
        ms_append_candidates(cmask != 0, s_coff, s_ccap, s_rc, s_rc2, s_rbase, k_var, cnt,
                             blockIdx.x & (CAND_SUB - 1), cand,
                             [&](auto&& f) {
#pragma unroll
                                 for (uint32_t u = 0; u < U; ++u) {
                                     const uint32_t j = (q0 + 64u * u) * 4;
                                     const uint32_t vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                                     for (uint32_t q = 0; q < 4; ++q)
                                         if (cmask & (1u << (4 * u + q)))
                                             f(vv[q], g0 + j + q,
                                               ((jj[u] >> (8 * q)) & 0xffu) - 1u + ((bmask >> (4 * u + q)) & 1u));
                                 }
                             });
    } else {
        for (uint32_t j0 = 0; j0 < n; j0 += BLOCK) {
            const uint32_t j = j0 + threadIdx.x;
            if (j < n) {
                const uint32_t bits = __float_as_uint(src[j]);
                bool is_cand, below_mid;
                const uint32_t jr = classify(bits, is_cand, below_mid);
                uint32_t level = 0;
                for (uint32_t k = 0; k < k_all; ++k) {
                    const bool keep = s_rv[k] < (int32_t)jr;
                    level += keep ? 1u : 0u;
                    if (w_out)
                        w_out[(uint64_t)k * w_stride + T.offset + e0 + j] = keep ? __uint_as_float(bits) : 0.0f;
                    if (want_mask) mask[(uint64_t)k * mask_stride + T.gbase + e0 + j] = keep ? 1 : 0;
                }
                if (is_cand) {
                    const uint32_t cl = jr - 1u + (below_mid ? 1u : 0u);
                    const uint32_t csb = blockIdx.x & (CAND_SUB - 1);
                    const uint32_t pos = atomicAdd(mcnt_cand(cnt, cl, csb), 1u);
                    const uint32_t cap = s_ccap[cl];
                    if (pos < cap) cand[(size_t)s_coff[cl] + (size_t)csb * cap + pos] = make_uint2(bits, g0 + j);
                } else {
                    mark(j, bits, level);
                }
            }
        }
    }
    for (uint32_t d = 32; d > 0; d >>= 1) nan |= __shfl_down(nan, d, 64);
    if (lane == 0 && nan) s_nan = 1;
    __syncthreads();
    // column sums: four threads per j, a quarter of the columns each
    if (ranked && threadIdx.x < 4 * (k_var + 1)) {
        const uint32_t j = threadIdx.x >> 2, q = threadIdx.x & 3u;
        uint32_t c = 0;
        for (uint32_t i = 0; i < BLOCK / 4; ++i) c += s_col[j * BLOCK + ((i * 4 + q + j) & (BLOCK - 1))];
        if (c) atomicAdd(mcnt_below(cnt, j, sb), c);
    }
    if (threadIdx.x == 0 && s_nan) atomicOr(&ms->status, 2u);
    // levels of the tile's filters and input features
    const uint32_t row_first = e0 / T.row_len;
    for (uint32_t s = threadIdx.x; s < nrows; s += BLOCK) {
        const uint32_t l = rowmax[s];
        if (l) {
            uint32_t* f = out_level + T.out_flag_off + row_first + s;
            if (*f < l) atomicMax(f, l);
        }
    }
    const uint32_t bfeat = (e0 / T.khw) % T.in_ch;
    for (uint32_t s = threadIdx.x; s < ncols; s += BLOCK) {
        const uint32_t l = colmax[s];
        if (l) {
            uint32_t* f = in_level + T.in_flag_off + mod_small(bfeat + s, T.in_ch, T.magic_in);
            if (*f < l) atomicMax(f, l);
        }
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

// Settles the candidates of ms_fused_kernel with the exact cuts: the pass wrote a
// candidate of ranks [a, j) as kept in all of them but the last, and in rank j - 1 iff
// key >= mid_{j-1}; here it is rewritten in every rank where that was the wrong side of
// the exact cut, and its level (variants that keep it: those that remove nothing, the
// ranks below a, and the ranks of [a, j) that keep it) goes into the level arrays.
// blockIdx.x: part of the region, blockIdx.y: rank (only a cluster's last rank owns a
// region), blockIdx.z: which of gridDim.z interleaved slices of the part.
__global__ __launch_bounds__(BLOCK) void ms_fixup_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ ranked_ids, uint32_t n_ranked,
    const MultiState* __restrict__ ms, const uint32_t* __restrict__ cnt,
    const uint2* __restrict__ cand, const shifter_threshold* __restrict__ thr,
    uint32_t n_zero, float* __restrict__ w_out, uint64_t w_stride, uint8_t* __restrict__ mask,
    uint64_t mask_stride, uint32_t* out_level, uint32_t* in_level) {
    constexpr uint32_t LDS_T = 1024;
    __shared__ uint32_t s_gbase[LDS_T];
    __shared__ uint32_t s_lo[MAXK + 1], s_hi[MAXK + 1], s_mid[MAXK], s_perm[MAXK];
    __shared__ uint64_t s_cut[MAXK];
    if (ms->status & 1u) return;
    const uint32_t cl = blockIdx.y, sb = blockIdx.x;
    if (ms->clast[cl] != cl) return;
    const uint32_t cap = ms->cand_cap[cl];
    const uint32_t n = min(cnt[((size_t)(MAXK + 1u + cl) * SPEC_SUB + sb) * 32u], cap);
    if (n == 0) return;
    const uint2* src = cand + (size_t)ms->cand_off[cl] + (size_t)sb * cap;
    const uint32_t k_var = ms->k;
    const bool in_lds = n_ranked <= LDS_T;
    if (in_lds)
        for (uint32_t i = threadIdx.x; i < n_ranked; i += BLOCK)
            s_gbase[i] = (uint32_t)tens[ranked_ids[i]].gbase;
    if (threadIdx.x <= MAXK) {
        s_lo[threadIdx.x] = threadIdx.x < MAXK ? ms->lo[threadIdx.x] : 0xffffffffu;
        s_hi[threadIdx.x] = threadIdx.x < MAXK ? ms->hi[threadIdx.x] : 0xffffffffu;
    }
    if (threadIdx.x < k_var) {
        s_perm[threadIdx.x] = ms->perm[threadIdx.x];
        s_cut[threadIdx.x] = thr[ms->perm[threadIdx.x]].cut;
        s_mid[threadIdx.x] = ms->mid[threadIdx.x];
    }
    __syncthreads();
    auto settle = [&](uint2 c) {
        const uint32_t key = c.x & 0x7fffffffu;
        uint32_t ka, kb;
        rank_range(s_lo, s_hi, key, &ka, &kb);
        kb = min(kb, k_var);
        const uint64_t comp = ((uint64_t)key << 32) | c.y;
        uint32_t a = 0, b = n_ranked;   // tensor holding global index c.y
        while (b - a > 1) {
            const uint32_t m2 = (a + b) >> 1;
            const uint32_t gb = in_lds ? s_gbase[m2] : (uint32_t)tens[ranked_ids[m2]].gbase;
            if (gb <= c.y) a = m2; else b = m2;
        }
        const DevTensor& T = tens[ranked_ids[a]];
        const uint32_t e = c.y - (uint32_t)T.gbase;
        uint32_t level = n_zero + ka;
        for (uint32_t r = ka; r < kb; ++r) {
            const bool removed = comp < s_cut[r];
            const bool written_removed = r + 1 == kb && key < s_mid[r];
            if (removed != written_removed) {    // written on the wrong side of the exact cut
                const uint32_t v = s_perm[r];
                if (w_out) w_out[(uint64_t)v * w_stride + T.offset + e] = removed ? 0.0f : __uint_as_float(c.x);
                if (mask) mask[(uint64_t)v * mask_stride + c.y] = removed ? 0 : 1;
            }
            level += removed ? 0u : 1u;
        }
        if (key != 0 && level != 0) {
            uint32_t* f = out_level + T.out_flag_off + e / T.row_len;
            if (*f < level) atomicMax(f, level);
            f = in_level + T.in_flag_off + (e / T.khw) % T.in_ch;
            if (*f < level) atomicMax(f, level);
        }
    };
    // four pairs per thread and step, their loads in flight together
    constexpr uint32_t U = 4;
    for (uint32_t i0 = blockIdx.z * U * BLOCK; i0 < n; i0 += gridDim.z * U * BLOCK) {
        uint2 c[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t i = i0 + u * BLOCK + threadIdx.x;
            c[u] = i < n ? src[i] : make_uint2(0, 0);
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u)
            if (i0 + u * BLOCK + threadIdx.x < n) settle(c[u]);
    }
}

void launch_spec_multi(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                       const PruneCounts& sorted_p, const MultiPerm& perm, uint32_t k,
                       uint64_t zero_mask, shifter_threshold* d_thr, const FusedBatch* fb,
                       uint32_t* zero_ptr, uint32_t zero_n) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size();
    hipStream_t s = ctx->stream;
    if (k != 0) {
        ProfileScope ps(ctx, K_SPEC_SAMPLE);
        // adds to the sample histogram, which every ranking leaves cleared; clears this
        // ranking's counters on the way
        SampleZero z;
        z.cnt = b.multi_cnt; z.k = k; z.ghist = b.multi_hist; z.list_cnt = b.multi_list_cnt;
        z.rout = b.multi->rout;
        if (fb) {       // the fused pass adds to the level arrays
            z.extra = b.levels;
            z.extra_n = (uint32_t)(m->info.sum_out_ch + m->info.sum_in_ch);
        }
        launch_spec_sample(ctx, m, d_w, z);
    } else if (fb) {
        launch_zero_levels(ctx, m);
    }
    {
        ProfileScope ps(ctx, K_SPEC_PREDICT);
        ms_predict_kernel<<<1, PREDICT_THREADS, 0, s>>>(
            b.multi, b.shist, b.multi_cnt, sorted_p, perm, k, m->sample_size, zero_mask, d_thr,
            b.dev_multi_rec, m->info.n_prunable, ctx->margin_sigmas, b.multi_tab, b.cand_cap_sb);
    }
    if (k == 0 && !fb) {         // every count was zero: no pass, which would have cleared zero_ptr
        if (zero_ptr) launch_zero_levels(ctx, m);
        return;
    }
    const bool nt = m->info.w_extent * 4 > (192ull << 20);
    if (fb) {
        VariantRanks rv;
        for (uint32_t v = 0; v < MAXK; ++v) rv.r[v] = -1;
        for (uint32_t r = 0; r < k; ++r) rv.r[perm.v[r]] = (int32_t)r;
        ProfileScope ps(ctx, K_MASK_SCAN_BATCH);
        // non-temporal hint as in the batched mask pass: only for cache-sized arenas
        auto kern = !nt ? ms_fused_kernel<true> : ms_fused_kernel<false>;
        kern<<<m->n_tiles, BLOCK, 0, s>>>(b.tens, b.tile_prefix, n_t, d_w, b.multi, b.multi_cnt, b.cand,
                                          rv, fb->k_all, fb->d_w_out, fb->w_stride,
                                          fb->d_mask, fb->mask_stride, b.levels,
                                          b.levels + m->info.sum_out_ch);
    } else {
        ProfileScope ps(ctx, K_SPEC_PASS);
        auto kern = nt ? ms_pass_kernel<true> : ms_pass_kernel<false>;
        kern<<<m->n_tiles, BLOCK, (k + 1) * BLOCK, s>>>(
            b.tens, b.tile_prefix, n_t, d_w, b.multi, b.multi_cnt, b.cand, b.multi_tab, zero_ptr, zero_n);
    }
    if (k != 0) {
        {
            ProfileScope ps(ctx, K_SPEC_FINISH);
            // CAND_SUB * 16 wavefronts in the extra layer cover the MAXK + 1 rows
            static_assert(CAND_SUB * (MF_THREADS / 64) >= MAXK + 1, "a wavefront per row of counters");
            ms_hist_kernel<<<dim3(CAND_SUB, k + 1), MF_THREADS, 0, s>>>(b.multi, b.multi_cnt, b.cand, b.multi_hist,
                                                                      b.multi_rowsum, k);
        }
        {
            ProfileScope ps(ctx, K_SPEC_FINISH2);
            ms_filter_kernel<<<dim3(CAND_SUB, k), MF_THREADS, 0, s>>>(b.multi, b.multi_cnt, b.cand, b.multi_hist,
                                                                     b.multi_rowsum, b.multi_list,
                                                                     b.multi_list_cnt);
        }
        {
            ProfileScope ps(ctx, K_SPEC_RANK);
            ms_rank_kernel<<<k, FIN_THREADS, 0, s>>>(b.multi, b.multi_list, b.multi_list_cnt, d_thr,
                                                     b.dev_multi_rec, b.dev_multi_status);
        }
    }
    if (fb) {
        if (k != 0) {
            ProfileScope ps(ctx, K_SPEC_FIXUP);
            ms_fixup_kernel<<<dim3(CAND_SUB, k, 16), BLOCK, 0, s>>>(
                b.tens, b.ranked_ids, m->n_ranked, b.multi, b.multi_cnt, b.cand, d_thr,
                fb->k_all - k, fb->d_w_out, fb->w_stride, fb->d_mask, fb->mask_stride, b.levels,
                b.levels + m->info.sum_out_ch);
        }
        if (!fb->levels_only) launch_expand_levels(ctx, m, d_thr, fb->k_all, fb->d_out_alive, fb->d_in_alive);
    }
}

}  // namespace shifter
