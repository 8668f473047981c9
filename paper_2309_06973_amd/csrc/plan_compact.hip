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

// One block per variant: sizes and offsets of every rebuilt tensor and vector (Algorithm 2, the
// "create new layer" step), tile prefix of the gather launch, capacity check.
// A rebuilt tensor is tiled in units of TILE floats of the OUTPUT ARENA starting at the
// 16-byte boundary at or below its first element, so that the gather stores whole
// aligned float4s; the ragged first and last quads are written element by element.
__global__ __launch_bounds__(BLOCK) void plan_kernel(
    const DevTensor* __restrict__ tens, uint32_t n_t, const DevVec* __restrict__ vecs,
    uint32_t n_v, const DevGroup* __restrict__ groups, uint32_t n_g,
    const uint32_t* __restrict__ new_width, uint64_t cap_w, uint64_t cap_v,
    PlanTensor* __restrict__ pt, PlanVec* __restrict__ pv, uint32_t* __restrict__ otp,
    PlanHeader* __restrict__ hdr) {
    __shared__ uint64_t smem[BLOCK / 64 + 1];
    __shared__ uint32_t s_collapse;
    // blockIdx.x = variant of a batch
    new_width += blockIdx.x * n_g;
    pt += blockIdx.x * n_t;
    pv += blockIdx.x * n_v;
    otp += blockIdx.x * (n_t + 1);
    hdr += blockIdx.x;
    if (threadIdx.x == 0) s_collapse = 0;
    uint64_t off = 0, tiles = 0, tot;
    for (uint32_t t0 = 0; t0 < n_t; t0 += BLOCK) {
        const uint32_t t = t0 + threadIdx.x;
        PlanTensor p;
        p.o2 = p.c2 = p.numel2 = p.pad = 0;
        if (t < n_t) {
            p.o2 = new_width[tens[t].out_group];
            p.c2 = new_width[tens[t].in_group];
            p.numel2 = p.o2 * p.c2 * tens[t].kk;
        }
        const uint64_t my_off = off + block_excl_scan_u64(p.numel2, smem, &tot);
        off += tot;
        const uint32_t span = p.numel2 ? (uint32_t)(my_off & 3u) + p.numel2 : 0;
        const uint32_t my_tiles = (span + TILE - 1) / TILE;
        const uint64_t my_tile0 = tiles + block_excl_scan_u64(my_tiles, smem, &tot);
        tiles += tot;
        if (t < n_t) {
            p.out_off = my_off;
            pt[t] = p;
            otp[t] = (uint32_t)my_tile0;
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
        otp[n_t] = (uint32_t)tiles;
        hdr->elems_w = off;
        hdr->elems_v = voff;
        hdr->total_tiles = (uint32_t)tiles;
        hdr->status = ((off > cap_w || voff > cap_v) ? 1u : 0u) | (s_collapse ? 2u : 0u);
    }
}

// Element (o', c', k) of a rebuilt tensor comes from (keep_out[o'], keep_in[c'], k) of the
// source, where k runs over the kk = kh * kw * in_mult elements of one (filter, channel)
// pair.  Blocks walk the output tiles; each thread fills aligned quads of the output
// arena (two divisions per quad, then incremental indices), and the blocks then share
// the per-channel vectors: v'[j] = v[keep[j]].
__global__ __launch_bounds__(BLOCK) void gather_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups, uint32_t n_t,
    const PlanTensor* __restrict__ pt, const uint32_t* __restrict__ otp,
    const PlanHeader* __restrict__ hdr, const float* __restrict__ w,
    const uint32_t* __restrict__ keep, float* __restrict__ w_out,
    const DevVec* __restrict__ vecs, uint32_t n_v, const PlanVec* __restrict__ pv,
    const float* __restrict__ v, float* __restrict__ v_out, uint64_t w_stride,
    uint64_t group_stride, uint64_t cap_w, uint64_t cap_v) {
    // blockIdx.y = variant of a batch
    pt += blockIdx.y * n_t;
    otp += blockIdx.y * (n_t + 1);
    hdr += blockIdx.y;
    pv += blockIdx.y * n_v;
    w += blockIdx.y * w_stride;
    keep += blockIdx.y * group_stride;
    w_out += blockIdx.y * cap_w;
    v_out += blockIdx.y * cap_v;
    if (hdr->status & 1u) return;
    const uint32_t total = hdr->total_tiles;
    for (uint32_t tile = blockIdx.x; tile < total; tile += gridDim.x) {
        const uint32_t t = find_tensor(otp, n_t, tile);
        const DevTensor T = tens[t];
        const PlanTensor P = pt[t];
        const uint32_t* keep_o = keep + groups[T.out_group].off;
        const uint32_t* keep_i = keep + groups[T.in_group].off;
        const uint32_t row2 = P.c2 * T.kk;
        const float* src = w + T.offset;
        // arena position of this tile's first quad, and of the tensor's ends
        const uint64_t a0 = (P.out_off & ~3ull) + (uint64_t)(tile - otp[t]) * TILE;
        const uint64_t begin = P.out_off, end = P.out_off + P.numel2;
        constexpr uint32_t U = TILE / BLOCK / 4;
        // phase 1: where each of this thread's quads starts in the rebuilt tensor
        uint64_t pq[U], first[U];
        uint32_t nv[U], o2[U], c2[U], k[U], ko[U], ki[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            pq[u] = a0 + 4ull * (threadIdx.x + BLOCK * u);
            nv[u] = 0;
            if (pq[u] >= end || pq[u] + 4 <= begin) continue;
            first[u] = pq[u] < begin ? begin : pq[u];
            nv[u] = (uint32_t)((pq[u] + 4 < end ? pq[u] + 4 : end) - first[u]);
            const uint32_t idx = (uint32_t)(first[u] - begin);
            o2[u] = idx / row2;
            const uint32_t rem = idx - o2[u] * row2;
            c2[u] = rem / T.kk;
            k[u] = rem - c2[u] * T.kk;
        }
        // phase 2: survivor indices of the quads' first elements (independent loads)
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            if (nv[u]) { ko[u] = keep_o[o2[u]]; ki[u] = keep_i[c2[u]]; }
        }
        // phase 3: the source elements; a quad crosses into the next channel or filter at
        // most a few times, each crossing costs one more index load
        float val[U][4];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            if (!nv[u]) continue;
            uint32_t oo = o2[u], cc = c2[u], kk2 = k[u];
            uint64_t so = (uint64_t)ko[u] * T.cin;
            uint64_t sc = (so + ki[u]) * T.kk;
#pragma unroll
            for (uint32_t c = 0; c < 4; ++c) {
                if (c < nv[u]) {
                    val[u][c] = src[sc + kk2];
                    if (++kk2 == T.kk) {
                        kk2 = 0;
                        if (++cc == P.c2) {
                            cc = 0;
                            ++oo;
                            if (oo < P.o2) so = (uint64_t)keep_o[oo] * T.cin;
                        }
                        if (oo < P.o2) sc = (so + keep_i[cc]) * T.kk;
                    }
                }
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            if (!nv[u]) continue;
            if (first[u] == pq[u] && nv[u] == 4) {
                *reinterpret_cast<float4*>(w_out + pq[u]) =
                    make_float4(val[u][0], val[u][1], val[u][2], val[u][3]);
            } else {
                for (uint32_t c = 0; c < nv[u]; ++c) w_out[first[u] + c] = val[u][c];
            }
        }
    }
    // the per-channel vectors, starting from the last blocks (those with no tile when
    // much was removed)
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
        // the tile counts are only known on the device: a fixed grid walks the tiles
        ProfileScope p(ctx, K_GATHER);
        const uint32_t bound = m->n_tiles + n_t;   // tiles when nothing is removed, at most
        const uint32_t per_variant = std::max(256u, ctx->hist_grid * 2 / k_var);
        const uint32_t grid = std::max(1u, std::min(bound, per_variant));
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
