// Exact multi-rank selection of the P-th smallest (|w|, g) pair: the unstructured
// magnitude ranking of Sec. II-A / Sec. III-C of the paper, done as a most-significant-
// digit radix select on the 31-bit magnitude keys (11 + 10 + 10 bits), followed by an
// index-ordered rank among the weights that tie with the threshold key.
//
// All ranks of a portfolio share the passes: round 0 builds one histogram; rounds 1
// and 2 histogram only the weights whose high bits match one of the (distinct)
// prefixes the ranks fell into, SLOTS_PER_PASS prefixes per pass over the arena.
#include "dev_common.h"

namespace shifter {

__global__ __launch_bounds__(BLOCK) void sel_init_kernel(SelState* st, uint32_t* ghist,
                                                         PruneCounts pc, uint32_t k) {
    const uint32_t tid = blockIdx.x * BLOCK + threadIdx.x;
    for (uint32_t i = tid; i < MAXK * HIST_BINS; i += gridDim.x * BLOCK) ghist[i] = 0;
    if (tid < MAXK) {
        SelRank r;
        r.rank = tid < k ? pc.p[tid] : 0;
        r.n_less = 0;
        r.n_equal = 0;
        r.prefix = 0;
        r.slot = 0;
        st->r[tid] = r;
        st->slot_prefix[tid] = 0;
    }
    if (tid == 0) {
        st->n_slots = 1;
        st->k = k;
        st->nan_seen = 0;
    }
}

// ROUND 0: bits 30..20 (2048 bins, every prunable weight).
// ROUND 1: bits 19..10, ROUND 2: bits 9..0 (1024 bins per prefix slot).
template <int ROUND>
__global__ __launch_bounds__(BLOCK) void hist_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    uint32_t n_t, uint32_t n_tiles, const float* __restrict__ w, SelState* st,
    uint32_t* ghist, uint32_t pass) {
    constexpr uint32_t NB = ROUND == 0 ? 2048u : 1024u;
    constexpr uint32_t SH = ROUND == 0 ? 20u : (ROUND == 1 ? 10u : 0u);
    constexpr uint32_t PSH = ROUND == 1 ? 20u : 10u;
    constexpr uint32_t SLOTS = ROUND == 0 ? 1u : SLOTS_PER_PASS;
    __shared__ uint32_t h[SLOTS * NB];

    uint32_t nsl = 1, first = 0;
    uint32_t pref[SLOTS];
    if (ROUND > 0) {
        const uint32_t total = st->n_slots;
        first = pass * SLOTS;
        if (first >= total) return;
        nsl = min(SLOTS, total - first);
#pragma unroll
        for (uint32_t j = 0; j < SLOTS; ++j)
            pref[j] = j < nsl ? st->slot_prefix[first + j] : 0xffffffffu;
    }
    for (uint32_t i = threadIdx.x; i < nsl * NB; i += BLOCK) h[i] = 0;
    __syncthreads();

    bool nan = false;
    auto add = [&](float x) {
        const uint32_t key = key_of(x);
        if (ROUND == 0) {
            nan |= key > 0x7f800000u;
            atomicAdd(&h[key >> SH], 1u);
        } else {
            const uint32_t p = key >> PSH, d = (key >> SH) & (NB - 1);
#pragma unroll
            for (uint32_t j = 0; j < SLOTS; ++j)
                if (p == pref[j]) atomicAdd(&h[j * NB + d], 1u);
        }
    };

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t t = find_tensor(tile_prefix, n_t, tile);
        if (!tens[t].prunable) continue;
        const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
        const uint32_t numel = tens[t].numel;
        const uint64_t off = tens[t].offset;
        const uint32_t n = min(TILE, numel - e0);
        const float* src = w + off + e0;
        if (n == TILE && (off & 3u) == 0) {
            const float4* s4 = reinterpret_cast<const float4*>(src);
            float4 v[TILE / BLOCK / 4];
#pragma unroll
            for (uint32_t u = 0; u < TILE / BLOCK / 4; ++u) v[u] = s4[threadIdx.x + BLOCK * u];
#pragma unroll
            for (uint32_t u = 0; u < TILE / BLOCK / 4; ++u) {
                add(v[u].x); add(v[u].y); add(v[u].z); add(v[u].w);
            }
        } else {
            for (uint32_t j = threadIdx.x; j < n; j += BLOCK) add(src[j]);
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < nsl * NB; i += BLOCK) {
        const uint32_t c = h[i];
        if (c) atomicAdd(&ghist[(first + i / NB) * HIST_BINS + (i % NB)], c);
    }
    if (ROUND == 0 && nan) st->nan_seen = 1;
}

// One block.  For every rank: locate the bin holding it in its slot's histogram,
// descend into that bin, then rebuild the slot table of distinct prefixes and clear the
// histograms for the next round.
__global__ __launch_bounds__(BLOCK) void select_kernel(SelState* st, uint32_t* ghist,
                                                       int round) {
    const uint32_t nb = round == 0 ? 2048u : 1024u;
    const uint32_t bits = round == 0 ? 11u : 10u;
    const uint32_t per = nb / BLOCK;   // 8 or 4 consecutive bins per thread
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t s_bin, s_cnt;
    __shared__ uint64_t s_less;
    const uint32_t k = st->k;
    for (uint32_t q = 0; q < k; ++q) {
        const uint64_t rank = st->r[q].rank;
        if (rank == 0) continue;
        const uint32_t* hist = ghist + st->r[q].slot * HIST_BINS;
        uint32_t c[8];
        uint64_t sum = 0;
        for (uint32_t j = 0; j < per; ++j) {
            c[j] = hist[threadIdx.x * per + j];
            sum += c[j];
        }
        uint64_t total;
        uint64_t base = block_excl_scan_u64(sum, smem, &total);
        if (base < rank && rank <= base + sum) {
            for (uint32_t j = 0; j < per; ++j) {
                if (rank <= base + c[j]) {
                    s_bin = threadIdx.x * per + j;
                    s_cnt = c[j];
                    s_less = base;
                    break;
                }
                base += c[j];
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            SelRank r = st->r[q];
            r.n_less += s_less;
            r.rank -= s_less;
            r.n_equal = s_cnt;
            r.prefix = (r.prefix << bits) | s_bin;
            st->r[q] = r;
        }
        __syncthreads();
    }
    // distinct prefixes -> slots (k <= 64: a quadratic de-duplication by one thread)
    if (threadIdx.x == 0) {
        uint32_t ns = 0;
        for (uint32_t q = 0; q < k; ++q) {
            if (st->r[q].rank == 0) continue;
            const uint32_t p = st->r[q].prefix;
            uint32_t s = 0;
            while (s < ns && st->slot_prefix[s] != p) ++s;
            if (s == ns) st->slot_prefix[ns++] = p;
            st->r[q].slot = s;
        }
        st->n_slots = ns;
    }
    for (uint32_t i = threadIdx.x; i < MAXK * HIST_BINS; i += BLOCK) ghist[i] = 0;
}

// After round 2 every slot prefix is a full key.  Count, per tile and per distinct
// key, the weights equal to it (index-ordered ranking of the ties needs these).
__global__ __launch_bounds__(BLOCK) void tie_count_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    uint32_t n_t, uint32_t n_tiles, const float* __restrict__ w,
    const SelState* __restrict__ st, uint32_t* __restrict__ tile_cnt) {
    __shared__ uint32_t s_cnt[MAXK];
    const uint32_t ns = st->n_slots;
    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t t = find_tensor(tile_prefix, n_t, tile);
        if (!tens[t].prunable) {
            for (uint32_t s = threadIdx.x; s < ns; s += BLOCK) tile_cnt[s * n_tiles + tile] = 0;
            continue;
        }
        for (uint32_t s = threadIdx.x; s < ns; s += BLOCK) s_cnt[s] = 0;
        __syncthreads();
        const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
        const uint32_t n = min(TILE, tens[t].numel - e0);
        const float* src = w + tens[t].offset + e0;
        for (uint32_t s = 0; s < ns; ++s) {
            const uint32_t key = st->slot_prefix[s];
            uint32_t c = 0;
            for (uint32_t j = threadIdx.x; j < n; j += BLOCK) c += key_of(src[j]) == key;
            // wave reduce, one LDS add per wave
            for (uint32_t d = 32; d > 0; d >>= 1) c += __shfl_down(c, d, 64);
            if ((threadIdx.x & 63u) == 0 && c) atomicAdd(&s_cnt[s], c);
        }
        __syncthreads();
        for (uint32_t s = threadIdx.x; s < ns; s += BLOCK) tile_cnt[s * n_tiles + tile] = s_cnt[s];
        __syncthreads();
    }
}

// One block per rank: find the tile, then the element, of the r-th weight (in index
// order) equal to the threshold key, and write the final record.
__global__ __launch_bounds__(BLOCK) void tie_final_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    uint32_t n_t, uint32_t n_tiles, const float* __restrict__ w,
    const SelState* __restrict__ st, const uint32_t* __restrict__ tile_cnt,
    PruneCounts pc, shifter_threshold* __restrict__ thr) {
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t s_tile, s_elem;
    __shared__ uint64_t s_rem;
    const uint32_t q = blockIdx.x;
    const SelRank r = st->r[q];
    shifter_threshold out;
    out.reserved = 0;
    out.n_prune = pc.p[q];
    if (r.rank == 0) {
        if (threadIdx.x == 0) {
            out.cut = 0; out.t_key = 0; out.g_cut = ~0ull; out.n_less = 0; out.n_equal = 0;
            thr[q] = out;
        }
        return;
    }
    if (threadIdx.x == 0) { s_tile = 0; s_rem = 1; s_elem = 0; }
    const uint32_t key = r.prefix;
    const uint32_t* cnt = tile_cnt + (uint64_t)r.slot * n_tiles;
    // 1. tile holding the r.rank-th equal weight
    const uint32_t chunk = (n_tiles + BLOCK - 1) / BLOCK;
    const uint32_t lo = min(n_tiles, threadIdx.x * chunk), hi = min(n_tiles, lo + chunk);
    uint64_t sum = 0;
    for (uint32_t i = lo; i < hi; ++i) sum += cnt[i];
    uint64_t total;
    uint64_t base = block_excl_scan_u64(sum, smem, &total);
    if (base < r.rank && r.rank <= base + sum) {
        for (uint32_t i = lo; i < hi; ++i) {
            const uint32_t c = cnt[i];
            if (r.rank <= base + c) { s_tile = i; s_rem = r.rank - base; break; }
            base += c;
        }
    }
    __syncthreads();
    // 2. element inside that tile: each thread owns TILE / BLOCK consecutive elements
    const uint32_t tile = s_tile;
    const uint64_t rem = s_rem;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, tens[t].numel - e0);
    const float* src = w + tens[t].offset + e0;
    constexpr uint32_t PER = TILE / BLOCK;
    const uint32_t j0 = threadIdx.x * PER;
    uint32_t c = 0;
    for (uint32_t j = j0; j < min(n, j0 + PER); ++j) c += key_of(src[j]) == key;
    uint64_t tot2;
    uint64_t b2 = block_excl_scan_u64(c, smem, &tot2);
    if (b2 < rem && rem <= b2 + c) {
        for (uint32_t j = j0; j < min(n, j0 + PER); ++j) {
            if (key_of(src[j]) == key && ++b2 == rem) { s_elem = j; break; }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint64_t g = tens[t].gbase + e0 + s_elem;
        out.t_key = key;
        out.g_cut = g;
        out.cut = (((uint64_t)key << 32) | g) + 1;
        out.n_less = r.n_less;
        out.n_equal = r.n_equal;
        thr[q] = out;
    }
}

// A flat run of n weights as a one-tensor model: filter 0 of a 1 x n linear layer at
// element 0, prunable, global index = element index.
__global__ void flat_tables_kernel(DevTensor* tens, uint32_t* tile_prefix, uint64_t n) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    DevTensor d;
    d.offset = 0;
    d.gbase = 0;
    d.numel = (uint32_t)n;
    d.out_ch = 1;
    d.in_ch = (uint32_t)n;
    d.khw = 1;
    d.row_len = (uint32_t)n;
    d.kk = 1;
    d.cin = (uint32_t)n;
    d.magic_khw = d.magic_row = d.magic_in = d.magic_kk = d.shift_kk = 0;
    d.out_group = 1;
    d.in_group = 0;
    d.out_flag_off = d.in_flag_off = 0;
    d.prunable = 1;
    d.band_rows = d.chunk_ch = d.src_chunks = 1;
    tens[0] = d;
    tile_prefix[0] = 0;
    tile_prefix[1] = (uint32_t)((n + TILE - 1) / TILE);
}

void launch_flat_tables(shifter_ctx* ctx, DevTensor* tens, uint32_t* tile_prefix, uint64_t n) {
    flat_tables_kernel<<<1, 64, 0, ctx->stream>>>(tens, tile_prefix, n);
}

void launch_select(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                   const PruneCounts& pc, uint32_t k, shifter_threshold* d_thr) {
    const auto& b = m->b;
    const SelectTables tb{b.tens, b.tile_prefix, (uint32_t)m->t.size(), m->n_tiles, b.sel, b.ghist,
                          b.tile_cnt};
    launch_select_tables(ctx, tb, d_w, pc, k, d_thr);
}

void launch_select_tables(shifter_ctx* ctx, const SelectTables& tb, const float* d_w,
                          const PruneCounts& pc, uint32_t k, shifter_threshold* d_thr) {
    const uint32_t n_t = tb.n_t, n_tiles = tb.n_tiles;
    const uint32_t grid = max(1u, min(n_tiles, ctx->hist_grid));
    hipStream_t s = ctx->stream;
    {
        ProfileScope p(ctx, K_SEL_INIT);
        sel_init_kernel<<<64, BLOCK, 0, s>>>(tb.sel, tb.ghist, pc, k);
    }
    {
        ProfileScope p(ctx, K_HIST0);
        hist_kernel<0><<<grid, BLOCK, 0, s>>>(tb.tens, tb.tile_prefix, n_t, n_tiles, d_w, tb.sel,
                                              tb.ghist, 0);
    }
    {
        ProfileScope p(ctx, K_SELECT);
        select_kernel<<<1, BLOCK, 0, s>>>(tb.sel, tb.ghist, 0);
    }
    const uint32_t passes = (k + SLOTS_PER_PASS - 1) / SLOTS_PER_PASS;
    for (uint32_t pass = 0; pass < passes; ++pass) {
        ProfileScope p(ctx, K_HIST1);
        hist_kernel<1><<<grid, BLOCK, 0, s>>>(tb.tens, tb.tile_prefix, n_t, n_tiles, d_w, tb.sel,
                                              tb.ghist, pass);
    }
    {
        ProfileScope p(ctx, K_SELECT);
        select_kernel<<<1, BLOCK, 0, s>>>(tb.sel, tb.ghist, 1);
    }
    for (uint32_t pass = 0; pass < passes; ++pass) {
        ProfileScope p(ctx, K_HIST2);
        hist_kernel<2><<<grid, BLOCK, 0, s>>>(tb.tens, tb.tile_prefix, n_t, n_tiles, d_w, tb.sel,
                                              tb.ghist, pass);
    }
    {
        ProfileScope p(ctx, K_SELECT);
        select_kernel<<<1, BLOCK, 0, s>>>(tb.sel, tb.ghist, 2);
    }
    {
        ProfileScope p(ctx, K_TIE_COUNT);
        tie_count_kernel<<<grid, BLOCK, 0, s>>>(tb.tens, tb.tile_prefix, n_t, n_tiles, d_w, tb.sel,
                                                tb.tile_cnt);
    }
    {
        ProfileScope p(ctx, K_TIE_FINAL);
        tie_final_kernel<<<k, BLOCK, 0, s>>>(tb.tens, tb.tile_prefix, n_t, n_tiles, d_w, tb.sel,
                                             tb.tile_cnt, pc, d_thr);
    }
}

}  // namespace shifter
