// Prune planner (Module 3 / Algorithm 1 of the paper, stated on channel groups) and
// model pruner (Module 4 / Algorithm 2): per-group survivor lists, then every tensor
// and per-channel vector gathered into its smaller dense shape.
#include <algorithm>

#include "dev_common.h"

namespace shifter {

// One block per group (and per variant of a batch).  alive[c] = frozen | OR over producers of out_alive[p][c];
// an exclusive scan of alive gives the old -> new map and the keep list.
__global__ __launch_bounds__(BLOCK) void propagate_kernel(
    const DevGroup* __restrict__ groups, const uint32_t* __restrict__ producers,
    const DevTensor* __restrict__ tens, const uint8_t* __restrict__ out_alive,
    uint32_t flags, uint8_t* __restrict__ group_alive, int32_t* __restrict__ index_map,
    uint32_t* __restrict__ keep, uint32_t* __restrict__ new_width, uint64_t out_alive_stride,
    uint64_t group_stride, uint32_t n_groups) {
    __shared__ uint32_t wave_cnt[BLOCK / 64];
    // blockIdx.y = variant of a batch
    out_alive += blockIdx.y * out_alive_stride;
    group_alive += blockIdx.y * group_stride;
    index_map += blockIdx.y * group_stride;
    keep += blockIdx.y * group_stride;
    new_width += blockIdx.y * n_groups;
    const DevGroup G = groups[blockIdx.x];
    const uint32_t n_prod = G.prod_end - G.prod_begin;
    const bool frozen = G.pinned || ((flags & SHIFTER_PAPER_FREEZE_RESIDUAL) && n_prod > 1);
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    uint32_t base = 0;
    for (uint32_t c0 = 0; c0 < G.width; c0 += BLOCK) {
        const uint32_t c = c0 + threadIdx.x;
        uint32_t a = 0;
        if (c < G.width) {
            a = frozen ? 1u : 0u;
            for (uint32_t p = G.prod_begin; p < G.prod_end && !a; ++p)
                a = out_alive[tens[producers[p]].out_flag_off + c] ? 1u : 0u;
        }
        const unsigned long long bal = __ballot(a);
        if (lane == 0) wave_cnt[wid] = (uint32_t)__popcll(bal);
        __syncthreads();
        uint32_t woff = 0, tot = 0;
        for (uint32_t i = 0; i < BLOCK / 64; ++i) {
            const uint32_t x = wave_cnt[i];
            if (i < wid) woff += x;
            tot += x;
        }
        const uint32_t pos = base + woff + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
        if (c < G.width) {
            group_alive[G.off + c] = (uint8_t)a;
            index_map[G.off + c] = a ? (int32_t)pos : -1;
            if (a) keep[G.off + pos] = c;
        }
        base += tot;
        __syncthreads();
    }
    for (uint32_t c = base + threadIdx.x; c < G.width; c += BLOCK) keep[G.off + c] = 0xffffffffu;
    if (threadIdx.x == 0) new_width[blockIdx.x] = base;
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
// the "create new layer" step), the work-unit prefix of the gather launch, capacity check.
// A gather work unit is a 2-D piece of one rebuilt tensor: GATHER_CHUNK consecutive
// columns (elements of a filter) times gather_unit_rows() rows (filters); for filters
// shorter than GATHER_CHUNK the wavefront's 1024 column slots hold several rows side by
// side (rows padded to a power of two, at least 64).  Every unit is four row steps deep.
__global__ __launch_bounds__(BLOCK) void plan_kernel(
    const DevTensor* __restrict__ tens, uint32_t n_t, const DevVec* __restrict__ vecs,
    uint32_t n_v, const DevGroup* __restrict__ groups, uint32_t n_g,
    const uint32_t* __restrict__ new_width, uint64_t cap_w, uint64_t cap_v,
    PlanTensor* __restrict__ pt, PlanVec* __restrict__ pv, uint32_t* __restrict__ oup,
    PlanHeader* __restrict__ hdr) {
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t s_collapse;
    // blockIdx.x = variant of a batch
    new_width += blockIdx.x * n_g;
    pt += blockIdx.x * n_t;
    pv += blockIdx.x * n_v;
    oup += blockIdx.x * (n_t + 1);
    hdr += blockIdx.x;
    if (threadIdx.x == 0) s_collapse = 0;
    uint64_t off = 0, units = 0, tot;
    for (uint32_t t0 = 0; t0 < n_t; t0 += BLOCK) {
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
        const uint64_t my_off = off + block_excl_scan_u64(p.numel2, smem, &tot);
        off += tot;
        const uint64_t my_unit0 = units + block_excl_scan_u64(my_units, smem, &tot);
        units += tot;
        if (t < n_t) {
            p.out_off = my_off;
            pt[t] = p;
            oup[t] = (uint32_t)my_unit0;
        }
    }
    uint64_t voff = 0;
    for (uint32_t v0 = 0; v0 < n_v; v0 += BLOCK) {
        const uint32_t v = v0 + threadIdx.x;
        PlanVec p;
        p.len2 = v < n_v ? new_width[vecs[v].group] : 0;
        p.pad = 0;
        p.out_off = voff + block_excl_scan_u64(p.len2, smem, &tot);
        voff += tot;
        if (v < n_v) pv[v] = p;
    }
    for (uint32_t g = threadIdx.x; g < n_g; g += BLOCK)
        if (new_width[g] == 0) s_collapse = 1;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t status = ((off > cap_w || voff > cap_v) ? 1u : 0u) | (s_collapse ? 2u : 0u);
        oup[n_t] = (uint32_t)units;
        hdr->elems_w = off;
        hdr->elems_v = voff;
        hdr->total_units = (status & 1u) ? 0u : (uint32_t)units;   // does not fit: gather nothing
        hdr->status = status;
    }
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

// Number of entries of the ascending list arr[0..n) that are below x, found by the whole
// wavefront: 64 evenly spaced probes per round narrow the range 64-fold, so lists of up
// to 4096 entries take two dependent loads.  Uniform result.
__device__ __forceinline__ uint32_t wave_lower_bound(const uint32_t* __restrict__ arr, uint32_t n,
                                                     uint32_t x, uint32_t lane) {
    uint32_t lo = 0, len = n;
    while (len > 0) {
        const uint32_t step = (len + 63u) >> 6;
        const uint32_t idx = lo + (lane + 1u) * step - 1u;
        const bool below = idx < lo + len && arr[idx] < x;
        const uint32_t c = (uint32_t)__popcll(__ballot(below));   // the probes below x are a prefix
        const uint32_t end = lo + len;
        lo += c * step;
        len = min(step - 1u, end - lo);
    }
    return lo;
}

// The rebuild of all K variants of a portfolio from one source, in source order.  A
// work unit is a rectangle of the SOURCE tensor - band_rows consecutive filters times
// chunk_ch consecutive input channels (about GATHER_CHUNK columns) - for one variant.
// What a variant keeps of the rectangle is a contiguous range of its keep lists (they
// are ascending; wave_lower_bound finds the ends), so the unit is an ordinary piece of
// the rebuilt tensor and gather_rows copies it.  The K units of a rectangle run in
// neighbouring blocks of the same XCD (blocks are dealt to the eight XCDs in turn;
// blocks 8 apart share one), each XCD working through a band of its own: a source line
// comes in from memory once and the other K - 1 variants find it in that XCD's L2.
__global__ __launch_bounds__(BLOCK) void gather_band_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups, uint32_t n_t,
    const PlanTensor* __restrict__ pt_all, const uint32_t* __restrict__ band_prefix,
    const PlanHeader* __restrict__ hdr_all, const float* __restrict__ w_all,
    const uint32_t* __restrict__ keep_all, float* __restrict__ w_out_all,
    const DevVec* __restrict__ vecs, uint32_t n_v, const PlanVec* __restrict__ pv_all,
    const float* __restrict__ v, float* __restrict__ v_out_all, uint64_t w_stride,
    uint64_t group_stride, uint64_t cap_w, uint64_t cap_v,
    const shifter_threshold* __restrict__ thr, uint32_t k_var, uint32_t k_blocks,
    uint32_t n_slots) {
    const uint32_t lane = threadIdx.x & 63u;
    // block -> (band within its group of eight = XCD, variant block, rectangle slot)
    const uint32_t x = blockIdx.x & 7u, j = blockIdx.x >> 3;
    const uint32_t slot = j / k_blocks, vb = j - slot * k_blocks;
    const uint32_t k = vb * (BLOCK / 64) + (threadIdx.x >> 6);
    if (slot < n_slots && k < k_var && !(hdr_all[k].status & 1u)) {
        const uint32_t t = find_tensor(band_prefix, n_t, slot);
        const DevTensor& T = tens[t];
        const PlanTensor P = pt_all[(uint64_t)k * n_t + t];
        const uint32_t local = slot - band_prefix[t];
        const uint32_t grp = local / T.src_chunks, chunk = local - grp * T.src_chunks;
        const uint32_t r0 = (grp * 8u + x) * T.band_rows;
        if (P.numel2 != 0 && r0 < T.out_ch) {
            const uint32_t* keep = keep_all + (uint64_t)k * group_stride;
            const uint32_t* keep_i = keep + groups[T.in_group].off;
            const uint32_t* keep_o = keep + groups[T.out_group].off;
            const uint32_t kk = T.kk;
            // surviving channels of the rectangle -> columns [col0, col0 + width) of the rebuilt filter
            const uint32_t ch0 = chunk * T.chunk_ch, ch1 = ch0 + T.chunk_ch;
            const uint32_t a0 = wave_lower_bound(keep_i, P.c2, ch0, lane);
            const uint32_t a1 = ch1 >= T.cin ? P.c2 : wave_lower_bound(keep_i, P.c2, ch1, lane);
            const uint32_t col0 = a0 * kk, width = (a1 - a0) * kk;
            // surviving filters of the band -> rows [row_begin, row_begin + n_rows)
            const uint32_t row_begin = wave_lower_bound(keep_o, P.o2, r0, lane);
            const uint32_t ko_lane = row_begin + lane < P.o2 ? keep_o[row_begin + lane] : 0xffffffffu;
            const uint32_t n_rows = (uint32_t)__popcll(__ballot(ko_lane < r0 + T.band_rows));
            if (width != 0 && n_rows != 0) {
                constexpr uint32_t U = GATHER_CHUNK / 64;
                const uint32_t lg = gather_cols_log2(width);
                uint32_t off[U], col[U], valid = 0;
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    const uint32_t e = (lane + 64 * u) & ((1u << lg) - 1);
                    valid |= (e < width ? 1u : 0u) << u;
                    const uint32_t r = col0 + min(e, width - 1);
                    col[u] = r;
                    const uint32_t c2 = kk == 1 ? r : div_u32(r, T.magic_kk, T.shift_kk);
                    off[u] = keep_i[c2] * kk + (r - c2 * kk);
                }
                const uint32_t row_end = row_begin + n_rows;
                const float* src = w_all + (uint64_t)k * w_stride + T.offset;
                float* dst = w_out_all + (uint64_t)k * cap_w + P.out_off;
                const uint64_t cut = (thr && T.prunable) ? thr[k].cut : 0;
                const uint32_t cut_key = (uint32_t)(cut >> 32), cut_g = (uint32_t)cut, gb = (uint32_t)T.gbase;
                switch (lg) {
                    case 10: gather_rows<10>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
                    case 9: gather_rows<9>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
                    case 8: gather_rows<8>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
                    case 7: gather_rows<7>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
                    default: gather_rows<6>(src, dst, ko_lane, off, col, valid, row_begin, row_end, T.row_len, P.row2, gb, cut_key, cut_g); break;
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
        for (uint32_t jv = threadIdx.x; jv < P.len2; jv += BLOCK) vo[P.out_off + jv] = v[V.offset + kp[jv]];
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
    propagate_kernel<<<dim3((uint32_t)m->g.size(), k_var), BLOCK, 0, ctx->stream>>>(
        b.groups, b.producers, b.tens, d_out_alive, flags, d_group_alive, d_index_map, d_keep,
        d_new_width, m->info.sum_out_ch, m->info.sum_group_width, (uint32_t)m->g.size());
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
                                                      b.plan_h);
    }
    {
        // the unit counts are only known on the device: the grid covers the case that
        // nothing is removed; wavefronts past the real count exit at once
        ProfileScope p(ctx, K_GATHER);
        if (d_thr && k_var > 1 && m->band_ok) {
            // K rebuilds from one shared source: source order, see gather_band_kernel
            // (measured: with K separate sparse arenas as the source there is nothing to
            // share and the output-ordered kernel below is the faster one)
            const uint32_t n_slots = m->band_prefix.back();
            const uint32_t k_blocks = (k_var + BLOCK / 64 - 1) / (BLOCK / 64);
            const uint32_t grid = std::max(1u, n_slots * k_blocks * 8u);
            gather_band_kernel<<<grid, BLOCK, 0, ctx->stream>>>(
                b.tens, b.groups, n_t, b.plan_t, b.band_prefix, b.plan_h, d_w, d_keep, d_w_out,
                b.vecs, n_v, b.plan_v, d_vecs, d_vecs_out, w_stride, m->info.sum_group_width,
                cap_w, cap_v, d_thr, k_var, k_blocks, n_slots);
            return;
        }
        const uint32_t grid = std::max(1u, (m->gather_units_bound + BLOCK / 64 - 1) / (BLOCK / 64));
        gather_kernel<<<dim3(grid, k_var), BLOCK, 0, ctx->stream>>>(
            b.tens, b.groups, n_t, b.plan_t, b.out_tile_prefix, b.plan_h, d_w, d_keep, d_w_out,
            b.vecs, n_v, b.plan_v, d_vecs, d_vecs_out, w_stride, m->info.sum_group_width, cap_w,
            cap_v, d_thr);
    }
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
