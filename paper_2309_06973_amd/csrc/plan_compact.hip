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
template <uint32_t LG>
__device__ __forceinline__ void gather_rows(const float* __restrict__ src, float* __restrict__ dst,
                                            uint32_t ko_lane,
                                            const uint32_t (&off)[GATHER_CHUNK / 64],
                                            const uint32_t (&col)[GATHER_CHUNK / 64],
                                            uint32_t row_begin, uint32_t row_end,
                                            uint32_t row_len, uint32_t row2) {
    constexpr uint32_t U = GATHER_CHUNK / 64;
    constexpr uint32_t ROWS_PAR = GATHER_CHUNK >> LG;   // rows side by side
    constexpr uint32_t UPR = U / ROWS_PAR;              // slot groups per row
    constexpr uint32_t RU = ROWS_PAR >= 4 ? 1 : 4 / ROWS_PAR;   // row steps in flight
    for (uint32_t row0 = row_begin; row0 < row_end; row0 += RU * ROWS_PAR) {
        float val[RU][U];
#pragma unroll
        for (uint32_t q = 0; q < RU; ++q) {
#pragma unroll
            for (uint32_t p = 0; p < ROWS_PAR; ++p) {
                const uint32_t row = row0 + q * ROWS_PAR + p;   // uniform
                if (row < row_end) {
                    const uint32_t ko = __builtin_amdgcn_readlane(ko_lane, row - row_begin);
                    const float* s = src + (uint64_t)ko * row_len;
#pragma unroll
                    for (uint32_t i = 0; i < UPR; ++i) {
                        const uint32_t u = p * UPR + i;
                        if (off[u] != 0xffffffffu) val[q][u] = s[off[u]];
                    }
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
                        if (off[u] != 0xffffffffu) d[col[u]] = val[q][u];
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
    uint64_t group_stride, uint64_t cap_w, uint64_t cap_v) {
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
        uint32_t off[U], col[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t slot = lane + 64 * u;
            const uint32_t r = chunk * GATHER_CHUNK + (slot & ((1u << lg) - 1));
            col[u] = r;
            off[u] = 0xffffffffu;
            if (r < P.row2) {
                const uint32_t c2 = kk == 1 ? r : div_u32(r, T.magic_kk, T.shift_kk);
                off[u] = keep_i[c2] * kk + (r - c2 * kk);
            }
        }
        const uint32_t row_begin = rblk * P.rb, row_end = min(P.o2, row_begin + P.rb);
        const uint32_t ko_lane = keep_o[min(row_begin + lane, row_end - 1)];
        const float* src = w + T.offset;
        float* dst = w_out + P.out_off;
        switch (lg) {
            case 10: gather_rows<10>(src, dst, ko_lane, off, col, row_begin, row_end, T.row_len, P.row2); break;
            case 9: gather_rows<9>(src, dst, ko_lane, off, col, row_begin, row_end, T.row_len, P.row2); break;
            case 8: gather_rows<8>(src, dst, ko_lane, off, col, row_begin, row_end, T.row_len, P.row2); break;
            case 7: gather_rows<7>(src, dst, ko_lane, off, col, row_begin, row_end, T.row_len, P.row2); break;
            default: gather_rows<6>(src, dst, ko_lane, off, col, row_begin, row_end, T.row_len, P.row2); break;
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
                    float* d_vecs_out, uint64_t cap_v, uint32_t k_var) {
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
        const uint32_t grid = std::max(1u, (m->gather_units_bound + BLOCK / 64 - 1) / (BLOCK / 64));
        gather_kernel<<<dim3(grid, k_var), BLOCK, 0, ctx->stream>>>(
            b.tens, b.groups, n_t, b.plan_t, b.out_tile_prefix, b.plan_h, d_w, d_keep, d_w_out,
            b.vecs, n_v, b.plan_v, d_vecs, d_vecs_out, w_stride, m->info.sum_group_width, cap_w,
            cap_v);
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
