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
//                  (P - n_below)-th candidate: a 65536-bin histogram of the candidate
//                  keys, one scan, and an exact rank inside the selected bin give the
//                  record; the fused form then fixes up the candidates only.
//
// The result is exact whenever step 4's check holds; otherwise (a sample that misled,
// an interval with too many ties, a full buffer) a status bit is raised and the host
// runs the multi-pass radix select instead.
#include "dev_common.h"

namespace shifter {

constexpr uint32_t SBINS = 65536;       // sample / candidate histogram bins
constexpr uint32_t SAMPLE_SHIFT = 15;   // sample bins: top 16 of the 31 key bits

__global__ __launch_bounds__(BLOCK) void spec_init_kernel(SpecState* ss, uint32_t* shist,
                                                          uint32_t* hist2, uint64_t p,
                                                          uint8_t* fa, uint64_t na,
                                                          uint8_t* fb, uint64_t nb) {
    const uint64_t tid = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * BLOCK;
    for (uint64_t i = tid; i < SBINS; i += stride) { shist[i] = 0; hist2[i] = 0; }
    for (uint64_t i = tid; i < na; i += stride) fa[i] = 0;
    for (uint64_t i = tid; i < nb; i += stride) fb[i] = 0;
    if (tid == 0) {
        ss->p = p;
        ss->n_below = 0;
        ss->n_inside = 0;
        ss->n_cand = 0;
        ss->m_valid = 0;
        ss->status = 0;
        ss->small_cnt = 0;
        ss->lo = 0;
        ss->hi = 0x7fffffffu;
        ss->sh = 15;
    }
}

// One wavefront per sampled tile: lanes 0..31 read line l0, lanes 32..63 line l0 + 64
// of the tile's 128 lines of 32 floats; l0 rotates with the tile index.
__global__ __launch_bounds__(BLOCK) void spec_sample_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    uint32_t n_t, uint32_t n_tiles, uint32_t tile_stride, const float* __restrict__ w,
    SpecState* ss, uint32_t* shist) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = blockIdx.x * (BLOCK / 64) + (threadIdx.x >> 6);
    const uint32_t n_waves = gridDim.x * (BLOCK / 64);
    uint32_t taken = 0;
    for (uint32_t s = wave; (uint64_t)s * tile_stride < n_tiles; s += n_waves) {
        const uint32_t tile = s * tile_stride;
        const uint32_t t = find_tensor(tile_prefix, n_t, tile);
        if (!tens[t].prunable) continue;
        const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
        const uint32_t n = min(TILE, tens[t].numel - e0);
        const uint32_t l0 = (tile * 37u) & 63u;
        const uint32_t j = (l0 + (lane >> 5) * 64u) * 32u + (lane & 31u);
        if (j < n) {
            const uint32_t key = key_of(w[tens[t].offset + e0 + j]);
            atomicAdd(&shist[key >> SAMPLE_SHIFT], 1u);
            ++taken;
        }
    }
    for (uint32_t d = 32; d > 0; d >>= 1) taken += __shfl_down(taken, d, 64);
    if (lane == 0 && taken) atomicAdd(&ss->m_valid, taken);
}

// One block: inclusive prefix of the sample histogram, then the candidate interval.
__global__ __launch_bounds__(BLOCK) void spec_predict_kernel(SpecState* ss,
                                                             const uint32_t* __restrict__ shist,
                                                             uint32_t* sprefix,
                                                             uint64_t n_prunable) {
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    constexpr uint32_t PER = SBINS / BLOCK;
    const uint32_t b0 = threadIdx.x * PER;
    uint64_t sum = 0;
    for (uint32_t i = 0; i < PER; ++i) sum += shist[b0 + i];
    uint64_t total;
    uint64_t run = block_excl_scan_u64(sum, smem, &total);
    for (uint32_t i = 0; i < PER; ++i) {
        run += shist[b0 + i];
        sprefix[b0 + i] = (uint32_t)run;
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x != 0) return;
    const uint64_t p = ss->p;
    const uint32_t m = ss->m_valid;
    uint32_t lo = 0, hi = 0x7fffffffu;
    if (p > 0 && m >= 256 && n_prunable > 0) {
        const double frac = (double)p / (double)n_prunable;
        const double centre = frac * (double)m;
        // 24 standard deviations of a simple random sample: the sample is systematic and
        // clustered by lines, so its error can exceed the binomial one several times
        const double delta = 24.0 * sqrt((double)m * frac * (1.0 - frac)) + 16.0;
        const double r_lo = centre - delta, r_hi = centre + delta;
        // first bin whose inclusive prefix exceeds r (holds the r-th sample, 0-based)
        auto bin_of = [&](double r) -> uint32_t {
            const uint32_t target = (uint32_t)r;
            uint32_t a = 0, b = SBINS - 1;
            while (a < b) {
                const uint32_t mid = (a + b) >> 1;
                if (sprefix[mid] > target) b = mid; else a = mid + 1;
            }
            return a;
        };
        if (r_lo > 0.0) lo = bin_of(r_lo) << SAMPLE_SHIFT;
        if (r_hi < (double)(m - 1)) hi = ((bin_of(r_hi) + 1u) << SAMPLE_SHIFT) - 1u;
    }
    uint32_t sh = 0;
    while (((uint64_t)(hi - lo) >> sh) >= SBINS) ++sh;
    ss->lo = lo;
    ss->hi = hi;
    ss->sh = sh;
}

// The one pass over the arena.  FUSED also writes the sparse weights, the mask and the
// alive flags of every weight outside the candidate interval (candidates are written as
// kept and carry no flag yet; spec_fixup_kernel settles them).
template <bool FUSED>
__global__ __launch_bounds__(BLOCK) void spec_pass_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    uint32_t n_t, const float* __restrict__ w, SpecState* ss, uint2* __restrict__ cand,
    uint32_t cap, float* __restrict__ w_out, uint8_t* __restrict__ mask, uint8_t* out_alive,
    uint8_t* in_alive) {
    __shared__ uint8_t rowf[FUSED ? TILE + 16 : 16];
    __shared__ uint8_t colf[FUSED ? TILE + 16 : 16];
    __shared__ uint32_t s_below, s_inside, s_nan;

    const uint32_t tile = blockIdx.x;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    const DevTensor T = tens[t];
    if (!FUSED && !T.prunable) return;
    const bool ranked = T.prunable != 0 && ss->p != 0;   // P = 0: nothing is removed
    const uint32_t lo = ss->lo, hi = ss->hi;
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const uint32_t g0 = (uint32_t)(T.gbase + e0);
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t c0 = 0, r0 = 0, nrows = 0, ncols = 0;
    if (threadIdx.x == 0) { s_below = 0; s_inside = 0; s_nan = 0; }
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
        const bool removed = ranked && key < lo;
        is_cand = ranked && key >= lo && key <= hi;
        below += removed ? 1u : 0u;
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
        for (uint32_t u = 0; u < U; ++u) v[u] = s4[threadIdx.x + BLOCK * u];
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
                reinterpret_cast<uint4*>(dst)[threadIdx.x + BLOCK * u] = o;
                if (mdst)
                    reinterpret_cast<uint32_t*>(mdst)[threadIdx.x + BLOCK * u] =
                        k0 | (k1 << 8) | (k2 << 16) | (k3 << 24);
            }
        }
        // append this wavefront's candidates with one atomic
        if (__ballot(cmask != 0)) {
            const uint32_t c = __popc(cmask);
            uint32_t incl = c;
            for (uint32_t d = 1; d < 64; d <<= 1) {
                const uint32_t y = __shfl_up(incl, d, 64);
                if (lane >= d) incl += y;
            }
            const uint32_t wave_total = __shfl(incl, 63, 64);
            uint32_t base = 0;
            if (lane == 63) {
                base = atomicAdd(&ss->n_cand, wave_total);
                atomicAdd(&s_inside, wave_total);
            }
            base = __shfl(base, 63, 64);
            uint32_t pos = base + incl - c;
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t j = (threadIdx.x + BLOCK * u) * 4;
                const uint32_t vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    if (cmask & (1u << (4 * u + q))) {
                        if (pos < cap) cand[pos] = make_uint2(vv[q] & 0x7fffffffu, g0 + j + q);
                        ++pos;
                    }
                }
            }
        }
    } else {
        for (uint32_t j = threadIdx.x; j < n; j += BLOCK) {
            uint32_t k;
            bool q;
            const uint32_t bits = __float_as_uint(src[j]);
            const uint32_t o = one(j, bits, k, q);
            if (FUSED) {
                dst[j] = __uint_as_float(o);
                if (mdst) mdst[j] = (uint8_t)k;
            }
            const unsigned long long bal = __ballot(q);
            if (q) {
                const uint32_t leader = (uint32_t)__ffsll((long long)bal) - 1u;
                uint32_t base = 0;
                if (lane == leader) {
                    base = atomicAdd(&ss->n_cand, (uint32_t)__popcll(bal));
                    atomicAdd(&s_inside, (uint32_t)__popcll(bal));
                }
                base = __shfl(base, leader, 64);
                const uint32_t pos = base + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
                if (pos < cap) cand[pos] = make_uint2(bits & 0x7fffffffu, g0 + j);
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
        if (s_below) atomicAdd(&ss->n_below, s_below);
        if (s_inside) atomicAdd(&ss->n_inside, s_inside);
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

// Histogram of the candidate keys relative to lo (exact keys when sh == 0).
__global__ __launch_bounds__(BLOCK) void spec_hist2_kernel(const SpecState* __restrict__ ss,
                                                           const uint2* __restrict__ cand,
                                                           uint32_t cap, uint32_t* hist2) {
    const uint32_t n = min(ss->n_cand, cap);
    const uint32_t lo = ss->lo, sh = ss->sh;
    for (uint32_t i = blockIdx.x * BLOCK + threadIdx.x; i < n; i += gridDim.x * BLOCK)
        atomicAdd(&hist2[(cand[i].x - lo) >> sh], 1u);
}

// One block: the check that makes the result exact, then the bin holding the P-th pair.
__global__ __launch_bounds__(BLOCK) void spec_locate_kernel(SpecState* ss,
                                                            const uint32_t* __restrict__ hist2,
                                                            uint32_t cap) {
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    const uint64_t p = ss->p;
    if (p == 0) return;
    const uint64_t below = ss->n_below, inside = ss->n_inside;
    if (ss->n_cand > cap || !(below < p && p <= below + inside)) {
        if (threadIdx.x == 0) atomicOr(&ss->status, 1u);
        return;
    }
    const uint64_t r = p - below;
    constexpr uint32_t PER = SBINS / BLOCK;
    const uint32_t b0 = threadIdx.x * PER;
    uint64_t sum = 0;
    for (uint32_t i = 0; i < PER; ++i) sum += hist2[b0 + i];
    uint64_t total;
    uint64_t base = block_excl_scan_u64(sum, smem, &total);
    if (base < r && r <= base + sum) {
        for (uint32_t i = 0; i < PER; ++i) {
            const uint32_t c = hist2[b0 + i];
            if (r <= base + c) {
                ss->bin = b0 + i;
                ss->bin_cnt = c;
                ss->r2 = r - base;
                ss->less = below + base;
                if (c > SPEC_SMALL_CAP) atomicOr(&ss->status, 1u);
                break;
            }
            base += c;
        }
    }
}

// Candidates of the selected bin -> a small list.
__global__ __launch_bounds__(BLOCK) void spec_filter_kernel(SpecState* ss,
                                                            const uint2* __restrict__ cand,
                                                            uint32_t cap, uint2* small) {
    if (ss->p == 0 || (ss->status & 1u)) return;
    const uint32_t n = min(ss->n_cand, cap);
    const uint32_t lo = ss->lo, sh = ss->sh, bin = ss->bin;
    for (uint32_t i = blockIdx.x * BLOCK + threadIdx.x; i < n; i += gridDim.x * BLOCK) {
        const uint2 c = cand[i];
        if (((c.x - lo) >> sh) == bin) {
            const uint32_t pos = atomicAdd(&ss->small_cnt, 1u);
            if (pos < SPEC_SMALL_CAP) small[pos] = c;
        }
    }
}

// One block: exact rank inside the small list by counting, then the record.
__global__ __launch_bounds__(BLOCK) void spec_rank_kernel(SpecState* ss,
                                                          const uint2* __restrict__ small,
                                                          shifter_threshold* thr) {
    __shared__ uint64_t comp[SPEC_SMALL_CAP];
    __shared__ uint64_t s_sel;
    __shared__ uint32_t s_lt, s_eq;
    shifter_threshold out;
    out.reserved = 0;
    out.n_prune = ss->p;
    if (ss->p == 0) {
        if (threadIdx.x == 0) {
            out.cut = 0; out.t_key = 0; out.g_cut = ~0ull; out.n_less = 0; out.n_equal = 0;
            *thr = out;
        }
        return;
    }
    if (ss->status & 1u) return;
    const uint32_t n = min(ss->small_cnt, SPEC_SMALL_CAP);
    if (n != ss->bin_cnt) {   // cannot happen unless the buffers were disturbed
        if (threadIdx.x == 0) atomicOr(&ss->status, 1u);
        return;
    }
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK)
        comp[i] = ((uint64_t)small[i].x << 32) | small[i].y;
    if (threadIdx.x == 0) { s_lt = 0; s_eq = 0; s_sel = 0; }
    __syncthreads();
    const uint64_t want = ss->r2 - 1;   // 0-based rank among the list
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) {
        const uint64_t c = comp[i];
        uint32_t rank = 0;
        for (uint32_t f = 0; f < n; ++f) rank += comp[f] < c;
        if (rank == want) s_sel = c;    // composites are distinct: exactly one hit
    }
    __syncthreads();
    const uint64_t sel = s_sel;
    const uint32_t key = (uint32_t)(sel >> 32);
    uint32_t lt = 0, eq = 0;
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) {
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
        out.n_less = ss->less + s_lt;
        out.n_equal = s_eq;
        *thr = out;
    }
}

// Fused form only: settle the candidates that the pass wrote as kept.
__global__ __launch_bounds__(BLOCK) void spec_fixup_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ ranked_ids,
    uint32_t n_ranked, const SpecState* __restrict__ ss, const uint2* __restrict__ cand,
    uint32_t cap, const shifter_threshold* __restrict__ thr, float* __restrict__ w_out,
    uint8_t* __restrict__ mask, uint8_t* out_alive, uint8_t* in_alive) {
    if (ss->status & 1u) return;
    const uint32_t n = min(ss->n_cand, cap);
    const uint64_t cut = thr->cut;
    for (uint32_t i = blockIdx.x * BLOCK + threadIdx.x; i < n; i += gridDim.x * BLOCK) {
        const uint2 c = cand[i];
        // tensor holding global index c.y: last ranked tensor with gbase <= g
        uint32_t a = 0, b = n_ranked;
        while (b - a > 1) {
            const uint32_t mid = (a + b) >> 1;
            if (tens[ranked_ids[mid]].gbase <= c.y) a = mid; else b = mid;
        }
        const DevTensor& T = tens[ranked_ids[a]];
        const uint32_t e = c.y - (uint32_t)T.gbase;
        if ((((uint64_t)c.x << 32) | c.y) < cut) {
            w_out[T.offset + e] = 0.0f;
            if (mask) mask[c.y] = 0;
        } else if (c.x != 0) {
            uint8_t* f = out_alive + T.out_flag_off + e / T.row_len;
            if (*f == 0) *f = 1;
            f = in_alive + T.in_flag_off + (e / T.khw) % T.in_ch;
            if (*f == 0) *f = 1;
        }
    }
}

void launch_spec_select(shifter_ctx* ctx, const shifter_model* m, const float* d_w, uint64_t p,
                        shifter_threshold* d_thr, float* d_w_out, uint8_t* d_mask,
                        uint8_t* d_out_alive, uint8_t* d_in_alive) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size();
    const bool fused = d_w_out != nullptr;
    hipStream_t s = ctx->stream;
    const uint32_t tile_stride = m->n_tiles > 32768u ? m->n_tiles / 32768u : 1u;
    const uint32_t small_grid = ctx->hist_grid;
    {
        ProfileScope ps(ctx, K_SPEC_INIT);
        spec_init_kernel<<<128, BLOCK, 0, s>>>(b.spec, b.shist, b.hist2, p, d_out_alive,
                                               fused ? m->info.sum_out_ch : 0, d_in_alive,
                                               fused ? m->info.sum_in_ch : 0);
    }
    {
        ProfileScope ps(ctx, K_SPEC_SAMPLE);
        const uint32_t sampled = (m->n_tiles + tile_stride - 1) / tile_stride;
        const uint32_t grid = min(small_grid, (sampled + BLOCK / 64 - 1) / (BLOCK / 64));
        spec_sample_kernel<<<grid, BLOCK, 0, s>>>(b.tens, b.tile_prefix, n_t, m->n_tiles,
                                                  tile_stride, d_w, b.spec, b.shist);
    }
    {
        ProfileScope ps(ctx, K_SPEC_PREDICT);
        spec_predict_kernel<<<1, BLOCK, 0, s>>>(b.spec, b.shist, b.sprefix, m->info.n_prunable);
    }
    {
        ProfileScope ps(ctx, K_SPEC_PASS);
        if (fused)
            spec_pass_kernel<true><<<m->n_tiles, BLOCK, 0, s>>>(
                b.tens, b.tile_prefix, n_t, d_w, b.spec, b.cand, b.cand_cap, d_w_out, d_mask,
                d_out_alive, d_in_alive);
        else
            spec_pass_kernel<false><<<m->n_tiles, BLOCK, 0, s>>>(
                b.tens, b.tile_prefix, n_t, d_w, b.spec, b.cand, b.cand_cap, nullptr, nullptr,
                nullptr, nullptr);
    }
    {
        ProfileScope ps(ctx, K_SPEC_FINISH);
        spec_hist2_kernel<<<small_grid, BLOCK, 0, s>>>(b.spec, b.cand, b.cand_cap, b.hist2);
        spec_locate_kernel<<<1, BLOCK, 0, s>>>(b.spec, b.hist2, b.cand_cap);
        spec_filter_kernel<<<small_grid, BLOCK, 0, s>>>(b.spec, b.cand, b.cand_cap, b.small);
        spec_rank_kernel<<<1, BLOCK, 0, s>>>(b.spec, b.small, d_thr);
    }
    if (fused) {
        ProfileScope ps(ctx, K_SPEC_FIXUP);
        spec_fixup_kernel<<<small_grid, BLOCK, 0, s>>>(
            b.tens, b.ranked_ids, m->n_ranked, b.spec, b.cand, b.cand_cap, d_thr, d_w_out,
            d_mask, d_out_alive, d_in_alive);
    }
}

}  // namespace shifter
