// Prune planner (Module 3 / Algorithm 1 of the paper, stated on channel groups) and
// model pruner (Module 4 / Algorithm 2): per-group survivor lists, then every tensor
// and per-channel vector gathered into its smaller dense shape.
#include <algorithm>

#include "dev_common.h"

namespace shifter {

// One block per group (and per variant of a batch).  alive[c] = frozen | OR over producers of
// out_alive[p][c]; an exclusive scan of alive gives the old -> new map and the keep list.
// The producers' flag offsets are fetched once (two dependent loads each) and a channel's
// flags are then loaded side by side: the kernel is a handful of memory latencies long.
// 512 threads: a twenty-variant step of a residual network is a thousand blocks, which
// then fit the chip at once (measured 16 against 21 us there with 1024, 12 against 10 us
// on the ten variants of a plain chain of wide layers).
// Liveness of filter i of the whole model comes either from a variant's flag bytes
// (out_alive) or, in a portfolio step, straight from the level array of the batched mask
// pass: alive <=> level[i] > pos, pos = number of variants with a smaller cut.
constexpr uint32_t PROP_THREADS = 512, PROP_LDS_PRODUCERS = 64;

__device__ __forceinline__ void propagate_group(
    const DevGroup G, const uint32_t* __restrict__ producers, const DevTensor* __restrict__ tens,
    const uint8_t* __restrict__ out_alive, const uint32_t* __restrict__ out_level, uint32_t pos,
    uint32_t flags, uint8_t* __restrict__ group_alive, int32_t* __restrict__ index_map,
    uint32_t* __restrict__ keep, uint32_t* __restrict__ new_width_g, uint32_t* wave_cnt,
    uint32_t* s_flag_off, uint32_t* below = nullptr) {
    constexpr uint32_t WAVES = PROP_THREADS / 64;
    const uint32_t n_prod = G.prod_end - G.prod_begin;
    const bool frozen = G.pinned || ((flags & SHIFTER_PAPER_FREEZE_RESIDUAL) && n_prod > 1);
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    if (!frozen && threadIdx.x < min(n_prod, PROP_LDS_PRODUCERS))
        s_flag_off[threadIdx.x] = tens[producers[G.prod_begin + threadIdx.x]].out_flag_off;
    __syncthreads();
    auto alive_at = [&](uint32_t i) -> uint32_t {
        return out_level ? (out_level[i] > pos ? 1u : 0u) : (uint32_t)out_alive[i];
    };
    uint32_t base = 0;
    for (uint32_t c0 = 0; c0 < G.width; c0 += PROP_THREADS) {
        const uint32_t c = c0 + threadIdx.x;
        uint32_t a = 0;
        if (c < G.width) {
            a = frozen ? 1u : 0u;
            if (!frozen) {
                const uint32_t n_lds = min(n_prod, PROP_LDS_PRODUCERS);
                for (uint32_t p = 0; p < n_lds; ++p) a |= alive_at(s_flag_off[p] + c);
                for (uint32_t p = G.prod_begin + n_lds; p < G.prod_end && !a; ++p)
                    a = alive_at(tens[producers[p]].out_flag_off + c);
                a = a ? 1u : 0u;
            }
        }
        const unsigned long long bal = __ballot(a);
        if (lane == 0) wave_cnt[wid] = (uint32_t)__popcll(bal);
        __syncthreads();
        uint32_t woff = 0, tot = 0;
        for (uint32_t i = 0; i < WAVES; ++i) {
            const uint32_t x = wave_cnt[i];
            if (i < wid) woff += x;
            tot += x;
        }
        const uint32_t pos_c = base + woff + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
        if (c < G.width) {
            group_alive[G.off + c] = (uint8_t)a;
            index_map[G.off + c] = a ? (int32_t)pos_c : -1;
            if (a) keep[G.off + pos_c] = c;
            if (below) below[c] = pos_c;      // surviving channels below c
        }
        base += tot;
        __syncthreads();
    }
    for (uint32_t c = base + threadIdx.x; c < G.width; c += PROP_THREADS) keep[G.off + c] = 0xffffffffu;
    if (threadIdx.x == 0) {
        *new_width_g = base;
        if (below) below[G.width] = base;
    }
}

__global__ __launch_bounds__(PROP_THREADS) void propagate_kernel(
    const DevGroup* __restrict__ groups, const uint32_t* __restrict__ producers,
    const DevTensor* __restrict__ tens, const uint8_t* __restrict__ out_alive,
    uint32_t flags, uint8_t* __restrict__ group_alive, int32_t* __restrict__ index_map,
    uint32_t* __restrict__ keep, uint32_t* __restrict__ new_width, uint64_t out_alive_stride,
    uint64_t group_stride, uint32_t n_groups) {
    __shared__ uint32_t wave_cnt[PROP_THREADS / 64];
    __shared__ uint32_t s_flag_off[PROP_LDS_PRODUCERS];
    // blockIdx.y = variant of a batch
    propagate_group(groups[blockIdx.x], producers, tens, out_alive + blockIdx.y * out_alive_stride,
                    nullptr, 0, flags, group_alive + blockIdx.y * group_stride,
                    index_map + blockIdx.y * group_stride, keep + blockIdx.y * group_stride,
                    new_width + blockIdx.y * n_groups + blockIdx.x, wave_cnt, s_flag_off);
}

// log2 of the column slots one row takes in a gather work unit: 10 (all 1024) for rows of
// 1024 or more elements, else the row length rounded up to a power of two, at least 64.
__host__ __device__ __forceinline__ uint32_t gather_cols_log2(uint32_t row2) {
    uint32_t lg = 6;
    while (lg < 10 && (1u << lg) < row2) ++lg;
    return lg;
}

// Rows of one gather work unit: four steps of max(4, rows side by side) rows.
__host__ __device__ __forceinline__ uint32_t gather_unit_rows(uint32_t lg) {
    const uint32_t rows_par = GATHER_CHUNK >> lg;
    return 4u * (rows_par > 4u ? rows_par : 4u);
}

// One block per variant: sizes and offsets of every rebuilt tensor and vector (Algorithm 2,
// the step that creates the smaller layer), the work-unit prefix of the gather launch,
// capacity check.
// A gather work unit is a 2-D piece of one rebuilt tensor: GATHER_CHUNK consecutive
// columns (elements of a filter) times gather_unit_rows() rows (filters); for filters
// shorter than GATHER_CHUNK the wavefront's 1024 column slots hold several rows side by
// side (rows padded to a power of two, at least 64).  Every unit is four row steps deep.
// The records also go, packed per variant (header, tensors, vectors), to a mirror in
// pinned host memory, so that the host reads a plan without a copy on the stream.
template <uint32_t THREADS>
__device__ __forceinline__ void plan_variant(
    uint32_t k, const DevTensor* __restrict__ tens, uint32_t n_t, const DevVec* __restrict__ vecs,
    uint32_t n_v, uint32_t n_g, const uint32_t* new_width, uint64_t cap_w, uint64_t cap_v,
    PlanTensor* __restrict__ pt, PlanVec* __restrict__ pv, uint32_t* __restrict__ oup,
    PlanHeader* __restrict__ hdr, uint8_t* __restrict__ pack, uint64_t* smem, uint32_t* s_collapse) {
    new_width += k * n_g;
    pt += k * n_t;
    pv += k * n_v;
    oup += k * (n_t + 1);
    hdr += k;
    pack += (uint64_t)k * (sizeof(PlanHeader) + n_t * sizeof(PlanTensor) + n_v * sizeof(PlanVec));
    PlanHeader* pack_h = reinterpret_cast<PlanHeader*>(pack);
    PlanTensor* pack_t = reinterpret_cast<PlanTensor*>(pack + sizeof(PlanHeader));
    PlanVec* pack_v = reinterpret_cast<PlanVec*>(pack + sizeof(PlanHeader) + n_t * sizeof(PlanTensor));
    if (threadIdx.x == 0) *s_collapse = 0;
    uint64_t off = 0, units = 0, tot;
    for (uint32_t t0 = 0; t0 < n_t; t0 += THREADS) {
        const uint32_t t = t0 + threadIdx.x;
        PlanTensor p;
        p.o2 = p.c2 = p.numel2 = p.row2 = p.chunks = 0;
        p.rb = GATHER_ROWS;
        uint32_t my_units = 0;
        if (t < n_t) {
            p.o2 = new_width[tens[t].out_group];
            p.c2 = new_width[tens[t].in_group];
            p.row2 = p.c2 * tens[t].kk;
            p.numel2 = p.o2 * p.row2;
            if (p.numel2) {
                p.chunks = (p.row2 + GATHER_CHUNK - 1) / GATHER_CHUNK;
                p.rb = gather_unit_rows(gather_cols_log2(p.row2));
                my_units = p.chunks * ((p.o2 + p.rb - 1) / p.rb);
            }
        }
        const uint64_t my_off = off + block_excl_scan_u64<THREADS>(p.numel2, smem, &tot);
        off += tot;
        const uint64_t my_unit0 = units + block_excl_scan_u64<THREADS>(my_units, smem, &tot);
        units += tot;
        if (t < n_t) {
            p.out_off = my_off;
            pt[t] = p;
            pack_t[t] = p;
            oup[t] = (uint32_t)my_unit0;
        }
    }
    uint64_t voff = 0;
    for (uint32_t v0 = 0; v0 < n_v; v0 += THREADS) {
        const uint32_t v = v0 + threadIdx.x;
        PlanVec p;
        p.len2 = v < n_v ? new_width[vecs[v].group] : 0;
        p.pad = 0;
        p.out_off = voff + block_excl_scan_u64<THREADS>(p.len2, smem, &tot);
        voff += tot;
        if (v < n_v) {
            pv[v] = p;
            pack_v[v] = p;
        }
    }
    __syncthreads();
    for (uint32_t g = threadIdx.x; g < n_g; g += THREADS)
        if (new_width[g] == 0) *s_collapse = 1;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t status = ((off > cap_w || voff > cap_v) ? 1u : 0u) | (*s_collapse ? 2u : 0u);
        PlanHeader h;
        h.elems_w = off;
        h.elems_v = voff;
        h.total_units = (status & 1u) ? 0u : (uint32_t)units;   // does not fit: gather nothing
        h.status = status;
        oup[n_t] = (uint32_t)units;
        *hdr = h;
        *pack_h = h;
    }
}

__global__ __launch_bounds__(BLOCK) void plan_kernel(
    const DevTensor* __restrict__ tens, uint32_t n_t, const DevVec* __restrict__ vecs,
    uint32_t n_v, const DevGroup* __restrict__ groups, uint32_t n_g,
    const uint32_t* __restrict__ new_width, uint64_t cap_w, uint64_t cap_v,
    PlanTensor* __restrict__ pt, PlanVec* __restrict__ pv, uint32_t* __restrict__ oup,
    PlanHeader* __restrict__ hdr, uint8_t* __restrict__ pack) {
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t s_collapse;
    (void)groups;
    // blockIdx.x = variant of a batch
    plan_variant<BLOCK>(blockIdx.x, tens, n_t, vecs, n_v, n_g, new_width, cap_w, cap_v, pt, pv, oup, hdr,
                        pack, smem, &s_collapse);
}

// x / d for any 32-bit x with the (magic, shift) pair the host derived from d >= 2.
__device__ __forceinline__ uint32_t div_u32(uint32_t x, uint32_t magic, uint32_t shift) {
    const uint32_t q = __umulhi(x, magic);
    return (((x - q) >> 1) + q) >> shift;
}

// The row loop of one gather work unit, for rows taking 1 << LG of the wavefront's 1024
// column slots (so 1024 >> LG rows sit side by side).  With LG known at compile time the
// row of slot group u is known too.  Lane j of ko_lane holds keep_out[row_begin + j] (a
// unit has at most 64 rows), so a row's source index is a register read, not a load.
// Every slot has a readable source offset (slots past the row's end repeat a valid one)
// and bit u of `valid` says whether slot u is stored: the loads of a row step are
// straight-line code, all in flight before the first is used.
template <uint32_t LG>
__device__ __forceinline__ void gather_rows(const float* __restrict__ src, float* __restrict__ dst,
                                            uint32_t ko_lane,
                                            const uint32_t (&off)[GATHER_CHUNK / 64],
                                            const uint32_t (&col)[GATHER_CHUNK / 64],
                                            uint32_t valid, uint32_t row_begin, uint32_t row_end,
                                            uint32_t row_len, uint32_t row2, uint32_t gb,
                                            uint32_t cut_key, uint32_t cut_g) {
    constexpr uint32_t U = GATHER_CHUNK / 64;
    constexpr uint32_t ROWS_PAR = GATHER_CHUNK >> LG;   // rows side by side
    constexpr uint32_t UPR = U / ROWS_PAR;              // slot groups per row
    constexpr uint32_t RU = ROWS_PAR >= 4 ? 1 : 4 / ROWS_PAR;   // row steps in flight
    for (uint32_t row0 = row_begin; row0 < row_end; row0 += RU * ROWS_PAR) {
        float val[RU][U];
        uint32_t g_row[RU][ROWS_PAR];
#pragma unroll
        for (uint32_t q = 0; q < RU; ++q) {
#pragma unroll
            for (uint32_t p = 0; p < ROWS_PAR; ++p) {
                // rows past the unit's end re-read its last row and are not stored
                const uint32_t row = min(row0 + q * ROWS_PAR + p, row_end - 1);   // uniform
                const uint32_t ko = __builtin_amdgcn_readlane(ko_lane, row - row_begin);
                const float* s = src + (uint64_t)ko * row_len;
                g_row[q][p] = gb + ko * row_len;
#pragma unroll
                for (uint32_t i = 0; i < UPR; ++i) val[q][p * UPR + i] = s[off[p * UPR + i]];
            }
        }
        // a weight below the cut in the order (|w| bits, global index) is a masked one and
        // reads as zero (cut 0: nothing is masked)
        if (cut_key | cut_g) {
#pragma unroll
            for (uint32_t q = 0; q < RU; ++q) {
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    const uint32_t key = __float_as_uint(val[q][u]) & 0x7fffffffu;
                    const bool removed =
                        key < cut_key || (key == cut_key && g_row[q][u / UPR] + off[u] < cut_g);
                    val[q][u] = removed ? 0.0f : val[q][u];
                }
            }
        }
#pragma unroll
        for (uint32_t q = 0; q < RU; ++q) {
#pragma unroll
            for (uint32_t p = 0; p < ROWS_PAR; ++p) {
                const uint32_t row = row0 + q * ROWS_PAR + p;
                if (row < row_end) {
                    float* d = dst + (uint64_t)row * row2;
#pragma unroll
                    for (uint32_t i = 0; i < UPR; ++i) {
                        const uint32_t u = p * UPR + i;
                        if ((valid >> u) & 1u) d[col[u]] = val[q][u];
                    }
                }
            }
        }
    }
}

// Algorithm 2's copy of the surviving channels.  Column r of a rebuilt filter comes from
// column keep_in[r / kk] * kk + r % kk of the source filter, the same for every filter of
// the tensor.  One wavefront per work unit: each lane first turns its (up to sixteen)
// column slots into source column offsets, held in registers, then walks the unit's
// rows: row o' is a plain strided copy from source row keep_out[o'] - no per-element
// index is loaded on the way, every load and store instruction covers up to 256
// consecutive bytes of the output (and of the source wherever neighbouring channels both
// survive), and about four rows are in flight at a time.  (Measured: with an index load
// in front of each data load the same copy runs at about 3.3 TB/s instead of 5.6.)  The
// blocks then share the per-channel vectors: v'[j] = v[keep[j]].
__global__ __launch_bounds__(BLOCK) void gather_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups, uint32_t n_t,
    const PlanTensor* __restrict__ pt, const uint32_t* __restrict__ oup,
    const PlanHeader* __restrict__ hdr, const float* __restrict__ w,
    const uint32_t* __restrict__ keep, float* __restrict__ w_out,
    const DevVec* __restrict__ vecs, uint32_t n_v, const PlanVec* __restrict__ pv,
    const float* __restrict__ v, float* __restrict__ v_out, uint64_t w_stride,
    uint64_t group_stride, uint64_t cap_w, uint64_t cap_v,
    const shifter_threshold* __restrict__ thr) {
    // blockIdx.y = variant of a batch
    pt += blockIdx.y * n_t;
    oup += blockIdx.y * (n_t + 1);
    hdr += blockIdx.y;
    pv += blockIdx.y * n_v;
    w += blockIdx.y * w_stride;
    keep += blockIdx.y * group_stride;
    w_out += blockIdx.y * cap_w;
    v_out += blockIdx.y * cap_v;
    if (hdr->status & 1u) return;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t unit = blockIdx.x * (BLOCK / 64) + (threadIdx.x >> 6);
    if (unit < hdr->total_units) {
        const uint32_t t = find_tensor(oup, n_t, unit);
        const DevTensor& T = tens[t];
        const PlanTensor P = pt[t];
        const uint32_t local = unit - oup[t];
        const uint32_t rblk = local / P.chunks, chunk = local - rblk * P.chunks;
        const uint32_t kk = T.kk;
        const uint32_t* keep_i = keep + groups[T.in_group].off;
        const uint32_t* keep_o = keep + groups[T.out_group].off;
        constexpr uint32_t U = GATHER_CHUNK / 64;
        const uint32_t lg = gather_cols_log2(P.row2);      // column slots per row = 1 << lg
        // this lane's slots -> column r and source column offset (0xffffffff: no column)
        uint32_t off[U], col[U], valid = 0;
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t slot = lane + 64 * u;
            const uint32_t r = chunk * GATHER_CHUNK + (slot & ((1u << lg) - 1));
            col[u] = r;
            valid |= (r < P.row2 ? 1u : 0u) << u;
            const uint32_t rr = min(r, P.row2 - 1);
            const uint32_t c2 = kk == 1 ? rr : div_u32(rr, T.magic_kk, T.shift_kk);
            off[u] = keep_i[c2] * kk + (rr - c2 * kk);
        }
        const uint32_t row_begin = rblk * P.rb, row_end = min(P.o2, row_begin + P.rb);
        const uint32_t ko_lane = keep_o[min(row_begin + lane, row_end - 1)];
        const float* src = w + T.offset;
        float* dst = w_out + P.out_off;
        // thr given: w is the dense arena and the variant's mask is applied on the way
        const uint64_t cut = (thr && T.prunable) ? thr[blockIdx.y].cut : 0;
        const uint32_t cut_key = (uint32_t)(cut >> 32), cut_g = (uint32_t)cut, gb = (uint32_t)T.gbase;
        switch (lg) {
            case 10: gather_rows<10>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
            case 9: gather_rows<9>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
            case 8: gather_rows<8>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
            case 7: gather_rows<7>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
            default: gather_rows<6>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
        }
    }
    // the per-channel vectors, starting from the last blocks
    for (uint32_t vi = gridDim.x - 1 - blockIdx.x; vi < n_v; vi += gridDim.x) {
        const DevVec V = vecs[vi];
        const PlanVec P = pv[vi];
        const uint32_t* kp = keep + groups[V.group].off;
        for (uint32_t j = threadIdx.x; j < P.len2; j += BLOCK)
            v_out[P.out_off + j] = v[V.offset + kp[j]];
    }
}

// Row and column tables of the portfolio rebuild, per variant: for every band of
// band_rows source filters the number of surviving filters below its first one, and for
// every chunk of chunk_ch source channels the number of surviving channels below its
// first one (keep lists are ascending, so these are lower bounds).  What a variant keeps
// of a source rectangle is then the range between two neighbouring entries of each.
__device__ __forceinline__ void rect_table_entry(
    uint32_t i, uint32_t k, const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups,
    uint32_t n_t, const uint32_t* __restrict__ rowtab_prefix, const uint32_t* __restrict__ coltab_prefix,
    const uint32_t* keep_all, const uint32_t* new_width_all, uint64_t group_stride, uint32_t n_groups,
    uint32_t* __restrict__ rowtab, uint32_t* __restrict__ coltab) {
    const uint32_t n_row = rowtab_prefix[n_t], n_col = coltab_prefix[n_t];
    if (i >= n_row + n_col) return;
    const bool is_row = i < n_row;
    const uint32_t e = is_row ? i : i - n_row;
    const uint32_t* prefix = is_row ? rowtab_prefix : coltab_prefix;
    uint32_t lo = 0, hi = n_t;   // tensor of entry e
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (prefix[mid] <= e) lo = mid; else hi = mid;
    }
    const DevTensor& T = tens[lo];
    const uint32_t j = e - prefix[lo];
    const int32_t grp = is_row ? T.out_group : T.in_group;
    const uint32_t x = is_row ? min(j * T.band_rows, T.out_ch) : min(j * T.chunk_ch, T.cin);
    const uint32_t* keep = keep_all + k * group_stride + groups[grp].off;
    const uint32_t n = min(new_width_all[k * n_groups + grp], groups[grp].width);
    uint32_t a = 0, len = n;     // entries of keep[0..n) below x
    while (len > 0) {
        const uint32_t half = len >> 1;
        if (keep[a + half] < x) { a += half + 1; len -= half + 1; } else len = half;
    }
    (is_row ? rowtab + (uint64_t)k * n_row : coltab + (uint64_t)k * n_col)[e] = a;
}

__global__ __launch_bounds__(BLOCK) void rect_tables_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups, uint32_t n_t,
    const uint32_t* __restrict__ rowtab_prefix, const uint32_t* __restrict__ coltab_prefix,
    const uint32_t* __restrict__ keep_all, const uint32_t* __restrict__ new_width_all,
    uint64_t group_stride, uint32_t n_groups, uint32_t* __restrict__ rowtab,
    uint32_t* __restrict__ coltab) {
    rect_table_entry(blockIdx.x * BLOCK + threadIdx.x, blockIdx.y, tens, groups, n_t, rowtab_prefix,
                     coltab_prefix, keep_all, new_width_all, group_stride, n_groups, rowtab, coltab);
}

// The group planning of a portfolio step in one launch (Module 3 for every group and
// variant, and the tables of Module 4's rebuild).  blockIdx.y = variant.  Blocks
// 0 .. n_groups - 1 each plan one group and, for the portfolio rebuild, fill the row and
// column tables of the tensors around it.  With levels as the source of liveness the blocks
// from n_groups on expand them into the variant's flag bytes (the outputs of the batched
// mask pass, which nothing in this launch reads).  The rebuild plans, which need every
// group's new width, follow in plan_kernel: a rendezvous inside this launch (the last
// block of a variant going on after a device-wide fence) was measured at 250 us - such a
// fence writes back the whole L2 of the block's XCD, just filled by the mask pass.
struct PlanAllArgs {
    const DevGroup* groups; const uint32_t* producers; const DevTensor* tens; uint32_t n_t;
    const DevVec* vecs; uint32_t n_v; uint32_t n_groups;
    const uint8_t* out_alive;          // flag bytes of every variant, or nullptr: take levels
    const uint32_t* out_level; const uint32_t* in_level;
    MultiPerm pos;                     // with levels: variants that remove less than variant k
    uint64_t n_out, n_in;
    uint8_t* exp_out_alive; uint8_t* exp_in_alive;   // where the levels are expanded to (in: may be nullptr)
    uint32_t flags;
    uint8_t* group_alive; int32_t* index_map; uint32_t* keep; uint32_t* new_width;
    uint64_t group_stride;
    const uint32_t* rowtab_prefix; const uint32_t* coltab_prefix; uint32_t* rowtab; uint32_t* coltab;
    uint32_t want_tables;
    uint32_t* below;                   // scratch: per variant and group, width + 1 counts of survivors below a channel
    const uint32_t* cons_prefix; const uint32_t* consumers;
    uint32_t k_var;
};

__global__ __launch_bounds__(PROP_THREADS) void plan_all_kernel(const PlanAllArgs A) {
    __shared__ uint32_t wave_cnt[PROP_THREADS / 64];
    __shared__ uint32_t s_flag_off[PROP_LDS_PRODUCERS];
    const uint32_t k = blockIdx.y;
    const uint32_t pos = A.pos.v[k];
    if (blockIdx.x >= A.n_groups) {
        const uint64_t i = (uint64_t)(blockIdx.x - A.n_groups) * PROP_THREADS + threadIdx.x;
        if (i < A.n_out) A.exp_out_alive[(uint64_t)k * A.n_out + i] = A.out_level[i] > pos ? 1 : 0;
        if (i < A.n_in && A.exp_in_alive) A.exp_in_alive[(uint64_t)k * A.n_in + i] = A.in_level[i] > pos ? 1 : 0;
        return;
    }
    const DevGroup G = A.groups[blockIdx.x];
    uint32_t* below = A.want_tables ? A.below + k * (A.group_stride + A.n_groups) + G.off + blockIdx.x : nullptr;
    propagate_group(G, A.producers, A.tens,
                    A.out_alive ? A.out_alive + (uint64_t)k * A.n_out : nullptr,
                    A.out_alive ? nullptr : A.out_level, pos, A.flags,
                    A.group_alive + k * A.group_stride, A.index_map + k * A.group_stride,
                    A.keep + k * A.group_stride, A.new_width + k * A.n_groups + blockIdx.x, wave_cnt,
                    s_flag_off, below);
    if (A.want_tables) {
        // the row tables of the tensors that write this group and the column tables of those
        // that read it: the survivors below the first filter of every band and below the
        // first channel of every chunk, which the scan above has just counted.  The tensors
        // side by side: each table starts with a chain of dependent loads (the tensor's index,
        // its record, its table's place), and a residual group has a dozen tensors around it
        __syncthreads();
        const uint32_t n_row = A.rowtab_prefix[A.n_t], n_col = A.coltab_prefix[A.n_t];
        const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
        const uint32_t n_prod = G.prod_end - G.prod_begin;
        const uint32_t cons_begin = A.cons_prefix[blockIdx.x], n_cons = A.cons_prefix[blockIdx.x + 1] - cons_begin;
        // wavefronts per tensor: all sixteen shared out among few tensors, one each for many
        constexpr uint32_t WAVES = PROP_THREADS / 64;
        uint32_t share = 1;
        while (share * 2u * (n_prod + n_cons) <= WAVES) share *= 2u;
        for (uint32_t x = wid / share; x < n_prod + n_cons; x += WAVES / share) {
            const bool writes = x < n_prod;
            const uint32_t t = writes ? A.producers[G.prod_begin + x] : A.consumers[cons_begin + x - n_prod];
            const uint32_t step = writes ? A.tens[t].band_rows : A.tens[t].chunk_ch;
            const uint32_t limit = writes ? A.tens[t].out_ch : A.tens[t].cin;
            const uint32_t* prefix = writes ? A.rowtab_prefix : A.coltab_prefix;
            const uint32_t first = prefix[t], n_e = prefix[t + 1] - first;
            uint32_t* tab = writes ? A.rowtab + (uint64_t)k * n_row + first : A.coltab + (uint64_t)k * n_col + first;
            for (uint32_t j = (wid % share) * 64u + lane; j < n_e; j += share * 64u) tab[j] = below[min(j * step, limit)];
        }
    }
}

// Position of column c of a staged rectangle row in LDS: within each group of 128
// columns, column 4 i + j sits at 32 j + i, so lanes reading every fourth column (four
// consecutive outputs per lane) fall into different banks.
__device__ __forceinline__ uint32_t rect_swizzle(uint32_t c) {
    return (c & ~127u) | ((c & 3u) << 5) | ((c >> 2) & 31u);
}

typedef float float4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // dword-aligned

// What one variant keeps of a source rectangle (gather_rect_kernel).
struct RectVariant {
    uint32_t row_begin, n_rows;   // rows [row_begin, row_begin + n_rows) of the rebuilt tensor
    uint32_t width, row2;         // width columns from col0 on; row2 = its filter length
    uint32_t a0, n_ch;            // its surviving channels: entries [a0, a0 + n_ch) of the keep list
    uint64_t dst;                 // element offset of (row 0, col0) in the output arenas
    uint64_t cut;                 // 0: nothing masked
};

// The rebuild of all K variants of a portfolio from the dense arena in one read of it
// (Algorithm 2 for the whole portfolio; Sec. III-D Module 4: all channels in one operation).
// One block per source rectangle - band_rows filters times chunk_ch whole channels, at
// most RECT_ELEMS floats.  All threads stage the rectangle in LDS with 16-byte loads
// while the first K threads fetch what each variant keeps of it (rows [row_begin,
// +n_rows) and columns [col0, +width) of its rebuilt tensor, from the two tables).
// Then the block's wavefronts take the variants in turn (an LDS counter hands them out):
// a lane owns four consecutive output columns of four quad slots, works out their LDS
// positions once per variant from the keep list, and per row reads them, applies the
// variant's cut (removed <=> (|w| bits, global index) < cut) and stores 16 bytes.
// Narrow pieces put several rows into one step.  Against the dword gather this needs
// about an eighth of the vector-memory instructions per KB moved, which is what bounded
// that kernel.
// Threads of one gather_rect_kernel block.  The kernel is bound by how many loads and
// stores a compute unit keeps in flight, and its staging tile (not its registers) limits
// the blocks per unit, so wider blocks bring more waves for the same tile: 512 threads
// measured 6 % faster than 256 on the twenty-variant portfolio and 4 % on the ten-variant
// one; 1024 threads (one block per unit) were slower.
constexpr uint32_t GR_THREADS = 512;

__global__ __launch_bounds__(GR_THREADS) void gather_rect_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups, uint32_t n_t,
    const PlanTensor* __restrict__ pt_all, const uint32_t* __restrict__ rect_prefix,
    const uint32_t* __restrict__ rowtab_prefix, const uint32_t* __restrict__ coltab_prefix,
    const uint32_t* __restrict__ rowtab, const uint32_t* __restrict__ coltab,
    const PlanHeader* __restrict__ hdr_all, const float* __restrict__ w, uint64_t w_extent,
    const uint32_t* __restrict__ keep_all, float* __restrict__ w_out_all,
    const DevVec* __restrict__ vecs, uint32_t n_v, const PlanVec* __restrict__ pv_all,
    const float* __restrict__ v, float* __restrict__ v_out_all, uint64_t group_stride,
    uint64_t cap_w, uint64_t cap_v, const shifter_threshold* __restrict__ thr, uint32_t k_var,
    uint32_t n_rects) {
    __shared__ float tile[RECT_ELEMS];
    __shared__ RectVariant meta[MAXK];
    __shared__ uint32_t next_k;
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t t = 0;
    bool live = false;   // blocks past the last band of a tensor only help with the vectors
    if (blockIdx.x < n_rects) {
        t = find_tensor(rect_prefix, n_t, blockIdx.x);
        const uint32_t local = blockIdx.x - rect_prefix[t];
        live = (((local >> 3) / tens[t].src_chunks) * 8u + (local & 7u)) * tens[t].band_rows < tens[t].out_ch;
    }
    if (live) {
        const DevTensor& T = tens[t];
        // eight neighbouring blocks take the same chunk of eight neighbouring bands, so an
        // XCD (blocks 8 apart) walks one band chunk by chunk and the pieces of a rebuilt
        // filter meet in one L2 before they are written back
        const uint32_t local = blockIdx.x - rect_prefix[t];
        const uint32_t grp = (local >> 3) / T.src_chunks, chunk = (local >> 3) - grp * T.src_chunks;
        const uint32_t band = grp * 8u + (local & 7u);
        const uint32_t kk = T.kk, row_len = T.row_len;
        const uint32_t r0 = band * T.band_rows, nr = min(T.band_rows, T.out_ch - r0);
        const uint32_t ch0 = chunk * T.chunk_ch, nch = min(T.chunk_ch, T.cin - ch0);
        const uint32_t c_base = ch0 * kk, wsrc = nch * kk;
        const uint32_t wp = (T.chunk_ch * kk + 127u) & ~127u;   // LDS row stride
        const uint32_t off_out = groups[T.out_group].off, off_in = groups[T.in_group].off;
        const uint32_t g_base = (uint32_t)T.gbase + c_base;
        // what each variant keeps of the rectangle
        if (threadIdx.x < k_var) {
            const uint32_t k = threadIdx.x;
            const uint32_t n_rowtab = rowtab_prefix[n_t], n_coltab = coltab_prefix[n_t];
            const PlanTensor P = pt_all[(uint64_t)k * n_t + t];
            const uint32_t* rt = rowtab + (uint64_t)k * n_rowtab + rowtab_prefix[t] + band;
            const uint32_t* ct = coltab + (uint64_t)k * n_coltab + coltab_prefix[t] + chunk;
            const uint32_t rb = rt[0], re = rt[1], a0 = ct[0], a1 = ct[1];
            RectVariant M;
            M.row_begin = rb;
            M.width = (a1 - a0) * kk;
            M.n_rows = ((hdr_all[k].status & 1u) || P.numel2 == 0 || M.width == 0) ? 0u : re - rb;
            M.row2 = P.row2;
            M.a0 = a0;
            M.n_ch = a1 - a0;
            M.dst = (uint64_t)k * cap_w + P.out_off + (uint64_t)a0 * kk;
            M.cut = T.prunable ? thr[k].cut : 0;
            meta[k] = M;
        }
        if (threadIdx.x == 0) next_k = 0;
        // stage rows r0 .. r0 + nr, columns c_base .. c_base + wsrc: a row takes 1 << lgt
        // threads (16 bytes each), so the block covers GR_THREADS >> lgt rows per round.  The
        // loads of eight rounds go out back to back before the first is written to LDS (one
        // trip for all but the odd shapes that pad a row to twice its threads)
        {
            const uint32_t qpr = (wsrc + 3u) >> 2;
            uint32_t lgt = 0;
            while ((1u << lgt) < qpr) ++lgt;
            const uint32_t c = (threadIdx.x & ((1u << lgt) - 1u)) * 4u;
            const uint32_t rstep = GR_THREADS >> lgt;
            constexpr uint32_t S = 8;
            if (c < wsrc) {
                float* d = tile + rect_swizzle(c);
                for (uint32_t rb = threadIdx.x >> lgt; rb < nr; rb += S * rstep) {
                    float4_a4 x[S];
#pragma unroll
                    for (uint32_t i = 0; i < S; ++i) {
                        const uint32_t r = rb + i * rstep;
                        const uint64_t gi = T.offset + (uint64_t)(r0 + r) * row_len + c_base + c;
                        x[i] = float4_a4{0.0f, 0.0f, 0.0f, 0.0f};
                        if (r < nr && gi + 3 < w_extent) x[i] = *reinterpret_cast<const float4_a4*>(w + gi);
                    }
#pragma unroll
                    for (uint32_t i = 0; i < S; ++i) {
                        const uint32_t r = rb + i * rstep;
                        const uint64_t gi = T.offset + (uint64_t)(r0 + r) * row_len + c_base + c;
                        if (r < nr && gi + 3 >= w_extent) {   // the last floats of the arena
                            x[i].x = w[gi];
                            if (gi + 1 < w_extent) x[i].y = w[gi + 1];
                            if (gi + 2 < w_extent) x[i].z = w[gi + 2];
                        }
                    }
                    // columns c .. c + 3 share (c & ~127) and (c >> 2) & 31: positions 32 apart
#pragma unroll
                    for (uint32_t i = 0; i < S; ++i) {
                        const uint32_t r = rb + i * rstep;
                        if (r < nr) {
                            float* dr = d + r * wp;
                            dr[0] = x[i].x; dr[32] = x[i].y; dr[64] = x[i].z; dr[96] = x[i].w;
                        }
                    }
                }
            }
        }
        __syncthreads();

        for (;;) {
            uint32_t k = 0;
            if (lane == 0) k = atomicAdd(&next_k, 1u);
            k = uniform_u32(k);
            if (k >= k_var) break;
            // the record is the same for every lane: keep it in scalar registers
            const uint32_t n_rows = uniform_u32(meta[k].n_rows);
            if (n_rows == 0) continue;
            const uint32_t row_begin = uniform_u32(meta[k].row_begin);
            const uint32_t width = uniform_u32(meta[k].width);
            const uint32_t row2 = uniform_u32(meta[k].row2);
            const uint32_t a0 = uniform_u32(meta[k].a0);
            const uint32_t n_ch = uniform_u32(meta[k].n_ch);
            const uint64_t dst_off = uniform_u64(meta[k].dst);
            const uint64_t cut = uniform_u64(meta[k].cut);
            const uint32_t* keep = keep_all + k * group_stride;
            const uint32_t* keep_i = keep + off_in + a0;
            const uint32_t lrow_lane = keep[off_out + row_begin + min(lane, n_rows - 1u)] - r0;
            // quad slots: 256 per step; a row takes 1 << lgq of them
            const uint32_t quads = (width + 3u) >> 2;
            uint32_t lgq = 0;
            while ((1u << lgq) < quads) ++lgq;
            // this lane's quads: byte position in a staged row and column in the rectangle.
            // Every entry of the keep list the lane needs is fetched first, side by side, and
            // only then used: one trip to memory per variant (a load placed next to its use
            // made the compiler wait for each in turn, eight trips)
            uint32_t pos4[4][4], scol[4][4], e0[4], kv[4][4], ee[4][4], cc[4][4];
            if (kk >= 4) {
                // four consecutive columns lie in at most two surviving channels
#pragma unroll
                for (uint32_t u = 0; u < 4; ++u) {
                    e0[u] = ((lane + 64u * u) & ((1u << lgq) - 1u)) * 4u;
                    ee[u][0] = min(e0[u], width - 1u);
                    cc[u][0] = div_u32(ee[u][0], T.magic_kk, T.shift_kk);
                    kv[u][0] = keep_i[cc[u][0]];
                    kv[u][1] = keep_i[min(cc[u][0] + 1u, n_ch - 1u)];
                }
#pragma unroll
                for (uint32_t u = 0; u < 4; ++u) {
                    const uint32_t rem = ee[u][0] - cc[u][0] * kk;
                    const uint32_t base_a = (kv[u][0] - ch0) * kk;
                    const uint32_t base_b = (kv[u][1] - ch0) * kk - kk;
#pragma unroll
                    for (uint32_t j = 0; j < 4; ++j)
                        scol[u][j] = (rem + j >= kk ? base_b : base_a) + rem + j;
                }
            } else {
#pragma unroll
                for (uint32_t u = 0; u < 4; ++u) {
                    e0[u] = ((lane + 64u * u) & ((1u << lgq) - 1u)) * 4u;
#pragma unroll
                    for (uint32_t j = 0; j < 4; ++j) {
                        ee[u][j] = min(e0[u] + j, width - 1u);
                        cc[u][j] = kk == 1 ? ee[u][j] : div_u32(ee[u][j], T.magic_kk, T.shift_kk);
                        kv[u][j] = keep_i[cc[u][j]];
                    }
                }
#pragma unroll
                for (uint32_t u = 0; u < 4; ++u)
#pragma unroll
                    for (uint32_t j = 0; j < 4; ++j)
                        scol[u][j] = (kv[u][j] - ch0) * kk + (ee[u][j] - cc[u][j] * kk);
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u)
#pragma unroll
                for (uint32_t j = 0; j < 4; ++j) pos4[u][j] = rect_swizzle(scol[u][j]) * 4u;
            float* dst = w_out_all + dst_off;
            const unsigned char* tile_b = reinterpret_cast<const unsigned char*>(tile);
            if (lgq >= 6) {
                // wide piece: quad slot group u belongs to one row, everything about the
                // row is scalar
                const uint32_t rows_par = 256u >> lgq;
                for (uint32_t row0 = 0; row0 < n_rows; row0 += rows_par) {
#pragma unroll
                    for (uint32_t u = 0; u < 4; ++u) {
                        const uint32_t row = row0 + ((64u * u) >> lgq);
                        if (row < n_rows) {
                            const uint32_t lrow = __builtin_amdgcn_readlane(lrow_lane, row);
                            const unsigned char* trow = tile_b + lrow * wp * 4u;
                            const uint32_t g_row = g_base + (r0 + lrow) * row_len;
                            float x[4];
#pragma unroll
                            for (uint32_t j = 0; j < 4; ++j) {
                                const float y = *reinterpret_cast<const float*>(trow + pos4[u][j]);
                                const uint64_t comp = ((uint64_t)(__float_as_uint(y) & 0x7fffffffu) << 32) |
                                                      (g_row + scol[u][j]);
                                x[j] = comp < cut ? 0.0f : y;
                            }
                            float* d = dst + (uint64_t)(row_begin + row) * row2 + e0[u];
                            if (e0[u] + 4u <= width) {
                                float4_a4 o;
                                o.x = x[0]; o.y = x[1]; o.z = x[2]; o.w = x[3];
                                *reinterpret_cast<float4_a4*>(d) = o;
                            } else if (e0[u] < width) {
                                d[0] = x[0];
                                if (e0[u] + 1u < width) d[1] = x[1];
                                if (e0[u] + 2u < width) d[2] = x[2];
                            }
                        }
                    }
                }
            } else {
                // narrow piece: 64 >> lgq rows per slot group, the row differs by lane
                const uint32_t rows_par = 256u >> lgq;
                for (uint32_t row0 = 0; row0 < n_rows; row0 += rows_par) {
#pragma unroll
                    for (uint32_t u = 0; u < 4; ++u) {
                        const uint32_t row = row0 + ((lane + 64u * u) >> lgq);
                        const uint32_t lrow = __shfl(lrow_lane, min(row, n_rows - 1u));
                        const unsigned char* trow = tile_b + lrow * wp * 4u;
                        const uint32_t g_row = g_base + (r0 + lrow) * row_len;
                        float x[4];
#pragma unroll
                        for (uint32_t j = 0; j < 4; ++j) {
                            const float y = *reinterpret_cast<const float*>(trow + pos4[u][j]);
                            const uint64_t comp = ((uint64_t)(__float_as_uint(y) & 0x7fffffffu) << 32) |
                                                  (g_row + scol[u][j]);
                            x[j] = comp < cut ? 0.0f : y;
                        }
                        if (row < n_rows && e0[u] < width) {
                            float* d = dst + (uint64_t)(row_begin + row) * row2 + e0[u];
                            if (e0[u] + 4u <= width) {
                                float4_a4 o;
                                o.x = x[0]; o.y = x[1]; o.z = x[2]; o.w = x[3];
                                *reinterpret_cast<float4_a4*>(d) = o;
                            } else {
                                d[0] = x[0];
                                if (e0[u] + 1u < width) d[1] = x[1];
                                if (e0[u] + 2u < width) d[2] = x[2];
                            }
                        }
                    }
                }
            }
        }
    }
    // the per-channel vectors of every variant, starting from the last blocks
    for (uint32_t xv = gridDim.x - 1 - blockIdx.x; xv < n_v * k_var; xv += gridDim.x) {
        const uint32_t kv = xv / n_v, vi = xv - kv * n_v;
        if (hdr_all[kv].status & 1u) continue;
        const DevVec V = vecs[vi];
        const PlanVec P = pv_all[(uint64_t)kv * n_v + vi];
        const uint32_t* kp = keep_all + (uint64_t)kv * group_stride + groups[V.group].off;
        float* vo = v_out_all + (uint64_t)kv * cap_v;
        for (uint32_t jv = threadIdx.x; jv < P.len2; jv += GR_THREADS) vo[P.out_off + jv] = v[V.offset + kp[jv]];
    }
}

__global__ __launch_bounds__(BLOCK) void copy_kernel(const float4* __restrict__ src,
                                                     float4* __restrict__ dst, uint64_t n4) {
    const uint64_t base = (uint64_t)blockIdx.x * (TILE / 4);
#pragma unroll
    for (uint32_t u = 0; u < TILE / 4 / BLOCK; ++u) {
        const uint64_t i = base + threadIdx.x + BLOCK * u;
        if (i < n4) dst[i] = src[i];
    }
}

__global__ __launch_bounds__(BLOCK) void copy_tail_kernel(const float* __restrict__ src,
                                                          float* __restrict__ dst,
                                                          uint64_t begin, uint64_t n) {
    const uint64_t i = begin + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

void launch_propagate(shifter_ctx* ctx, const shifter_model* m, const uint8_t* d_out_alive,
                      uint32_t flags, uint8_t* d_group_alive, int32_t* d_index_map,
                      uint32_t* d_keep, uint32_t* d_new_width, uint32_t k_var) {
    const auto& b = m->b;
    ProfileScope p(ctx, K_PROPAGATE);
    propagate_kernel<<<dim3((uint32_t)m->g.size(), k_var), PROP_THREADS, 0, ctx->stream>>>(
        b.groups, b.producers, b.tens, d_out_alive, flags, d_group_alive, d_index_map, d_keep,
        d_new_width, m->info.sum_out_ch, m->info.sum_group_width, (uint32_t)m->g.size());
}

// Whether the rebuild of k_var variants takes the rectangle kernel (one read of a shared
// dense source) or the output-ordered gather.
static bool use_rect(const shifter_model* m, uint32_t k_var, const shifter_threshold* d_thr) {
    // a single variant gains nothing from a shared read: the rectangle kernel reads the whole
    // dense arena, the output-ordered gather only the rows and channels that survive
    // (measured at 95 % sparsity on 1.3 GB: 246 us against 45)
    return d_thr && k_var > 1 && m->rect_ok && m->rect_prefix.back() > 0;
}

// The gather launch alone; the plan (and, for the rectangle kernel, the tables) must be
// on the device already.
static void launch_gather(shifter_ctx* ctx, const shifter_model* m, const float* d_w, uint64_t w_stride,
                          const float* d_vecs, const uint32_t* d_keep, float* d_w_out, uint64_t cap_w,
                          float* d_vecs_out, uint64_t cap_v, uint32_t k_var,
                          const shifter_threshold* d_thr) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size(), n_v = (uint32_t)m->v.size();
    // the unit counts are only known on the device: the grid covers the case that
    // nothing is removed; wavefronts past the real count exit at once
    ProfileScope p(ctx, K_GATHER);
    if (use_rect(m, k_var, d_thr)) {
        const uint32_t n_rects = m->rect_prefix.back();
        gather_rect_kernel<<<std::max(1u, n_rects), GR_THREADS, 0, ctx->stream>>>(
            b.tens, b.groups, n_t, b.plan_t, b.rect_prefix, b.rowtab_prefix, b.coltab_prefix,
            b.rowtab, b.coltab, b.plan_h, d_w, m->info.w_extent, d_keep, d_w_out, b.vecs, n_v,
            b.plan_v, d_vecs, d_vecs_out, m->info.sum_group_width, cap_w, cap_v, d_thr, k_var,
            n_rects);
        return;
    }
    const uint32_t grid = std::max(1u, (m->gather_units_bound + BLOCK / 64 - 1) / (BLOCK / 64));
    gather_kernel<<<dim3(grid, k_var), BLOCK, 0, ctx->stream>>>(
        b.tens, b.groups, n_t, b.plan_t, b.out_tile_prefix, b.plan_h, d_w, d_keep, d_w_out,
        b.vecs, n_v, b.plan_v, d_vecs, d_vecs_out, w_stride, m->info.sum_group_width, cap_w,
        cap_v, d_thr);
}

void launch_compact(shifter_ctx* ctx, const shifter_model* m, const float* d_w, uint64_t w_stride,
                    const float* d_vecs, const uint32_t* d_keep,
                    const uint32_t* d_new_width, float* d_w_out, uint64_t cap_w,
                    float* d_vecs_out, uint64_t cap_v, uint32_t k_var,
                    const shifter_threshold* d_thr) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size(), n_v = (uint32_t)m->v.size();
    {
        ProfileScope p(ctx, K_PLAN);
        plan_kernel<<<k_var, BLOCK, 0, ctx->stream>>>(b.tens, n_t, b.vecs, n_v, b.groups,
                                                      (uint32_t)m->g.size(), d_new_width, cap_w,
                                                      cap_v, b.plan_t, b.plan_v, b.out_tile_prefix,
                                                      b.plan_h, b.dev_plan);
        if (use_rect(m, k_var, d_thr)) {
            // K rebuilds from one shared source: one read of it, see gather_rect_kernel
            // (with K separate sparse arenas as the source there is nothing to share and
            // the output-ordered kernel is used)
            const uint32_t n_tab = m->rowtab_prefix.back() + m->coltab_prefix.back();
            rect_tables_kernel<<<dim3((n_tab + BLOCK - 1) / BLOCK, k_var), BLOCK, 0, ctx->stream>>>(
                b.tens, b.groups, n_t, b.rowtab_prefix, b.coltab_prefix, d_keep, d_new_width,
                m->info.sum_group_width, (uint32_t)m->g.size(), b.rowtab, b.coltab);
        }
    }
    launch_gather(ctx, m, d_w, w_stride, d_vecs, d_keep, d_w_out, cap_w, d_vecs_out, cap_v, k_var, d_thr);
}

// Steps 4 and 5 of a portfolio step behind its mask pass: one planning launch (groups,
// rebuild plans, tables; with from_levels also the variants' flag bytes, expanded from the
// level arrays the batched mask pass left) and the gather.
void launch_plan_and_gather(shifter_ctx* ctx, const shifter_model* m, const PortfolioBuffers& a,
                            bool from_levels, const MultiPerm& pos) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size(), n_v = (uint32_t)m->v.size();
    const uint32_t n_g = (uint32_t)m->g.size();
    const uint64_t n_out = m->info.sum_out_ch, n_in = m->info.sum_in_ch;
    // the source of the rebuild: the dense arena masked on the way, unless only the sparse
    // arenas can serve the output-ordered gather
    const bool rect = use_rect(m, a.k_var, a.d_thr);
    PlanAllArgs A;
    A.groups = b.groups; A.producers = b.producers; A.tens = b.tens; A.n_t = n_t;
    A.vecs = b.vecs; A.n_v = n_v; A.n_groups = n_g;
    A.out_alive = from_levels ? nullptr : a.d_out_alive;
    A.out_level = b.levels; A.in_level = b.levels + n_out; A.pos = pos;
    A.n_out = n_out; A.n_in = n_in;
    A.exp_out_alive = a.d_out_alive; A.exp_in_alive = a.d_in_alive;
    A.flags = a.flags;
    A.group_alive = a.d_group_alive; A.index_map = a.d_index_map; A.keep = a.d_keep;
    A.new_width = a.d_new_width; A.group_stride = m->info.sum_group_width;
    A.rowtab_prefix = b.rowtab_prefix; A.coltab_prefix = b.coltab_prefix; A.rowtab = b.rowtab;
    A.coltab = b.coltab; A.want_tables = rect ? 1u : 0u;
    A.below = b.below; A.cons_prefix = b.cons_prefix; A.consumers = b.consumers;
    A.k_var = a.k_var;
    const uint64_t mx = std::max<uint64_t>(n_out > n_in ? n_out : n_in, 1);
    const uint32_t expand_blocks = from_levels ? (uint32_t)((mx + PROP_THREADS - 1) / PROP_THREADS) : 0u;
    {
        ProfileScope p(ctx, K_PROPAGATE);
        plan_all_kernel<<<dim3(n_g + expand_blocks, a.k_var), PROP_THREADS, 0, ctx->stream>>>(A);
    }
    {
        ProfileScope p(ctx, K_PLAN);
        plan_kernel<<<a.k_var, BLOCK, 0, ctx->stream>>>(b.tens, n_t, b.vecs, n_v, b.groups, n_g, a.d_new_width,
                                                        a.cap_w, a.cap_v, b.plan_t, b.plan_v,
                                                        b.out_tile_prefix, b.plan_h, b.dev_plan);
    }
    const bool dense_src = rect || !a.d_w_sparse;
    launch_gather(ctx, m, dense_src ? a.d_w : a.d_w_sparse, dense_src ? 0 : a.w_stride, a.d_vecs, a.d_keep,
                  a.d_w_out, a.cap_w, a.d_vecs_out, a.cap_v, a.k_var, dense_src ? a.d_thr : nullptr);
}

void launch_copy(shifter_ctx* ctx, const float* src, float* dst, uint64_t n) {
    const uint64_t n4 = n / 4;
    ProfileScope p(ctx, K_COPY);
    if (n4)
        copy_kernel<<<(uint32_t)((n4 + TILE / 4 - 1) / (TILE / 4)), BLOCK, 0, ctx->stream>>>(
            reinterpret_cast<const float4*>(src), reinterpret_cast<float4*>(dst), n4);
    if (n4 * 4 < n) copy_tail_kernel<<<1, BLOCK, 0, ctx->stream>>>(src, dst, n4 * 4, n);
}

}  // namespace shifter
