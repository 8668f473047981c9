// Prune planner (Module 3 / Algorithm 1 of the paper, stated on channel groups) and
// model pruner (Module 4 / Algorithm 2): per-group survivor lists, then every tensor
// and per-channel vector gathered into its smaller dense shape.
#include "dev_common.h"

namespace shifter {

// One block per group.  alive[c] = frozen | OR over producers of out_alive[p][c];
// an exclusive scan of alive gives the old -> new map and the keep list.
__global__ __launch_bounds__(BLOCK) void propagate_kernel(
    const DevGroup* __restrict__ groups, const uint32_t* __restrict__ producers,
    const DevTensor* __restrict__ tens, const uint8_t* __restrict__ out_alive,
    uint32_t flags, uint8_t* __restrict__ group_alive, int32_t* __restrict__ index_map,
    uint32_t* __restrict__ keep, uint32_t* __restrict__ new_width) {
    __shared__ uint32_t wave_cnt[BLOCK / 64];
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

// One block: sizes and offsets of every rebuilt tensor and vector (Algorithm 2, the
// "create new layer" step), tile prefix of the gather launch, capacity check.
__global__ __launch_bounds__(BLOCK) void plan_kernel(
    const DevTensor* __restrict__ tens, uint32_t n_t, const DevVec* __restrict__ vecs,
    uint32_t n_v, const DevGroup* __restrict__ groups, uint32_t n_g,
    const uint32_t* __restrict__ new_width, uint64_t cap_w, uint64_t cap_v,
    PlanTensor* __restrict__ pt, PlanVec* __restrict__ pv, uint32_t* __restrict__ otp,
    PlanHeader* __restrict__ hdr) {
    if (threadIdx.x != 0) return;
    uint64_t off = 0;
    uint32_t tiles = 0;
    for (uint32_t t = 0; t < n_t; ++t) {
        PlanTensor p;
        p.o2 = new_width[tens[t].out_group];
        p.c2 = new_width[tens[t].in_group];
        p.numel2 = p.o2 * p.c2 * tens[t].kk;
        p.out_off = off;
        p.pad = 0;
        pt[t] = p;
        otp[t] = tiles;
        off += p.numel2;
        tiles += (p.numel2 + TILE - 1) / TILE;
    }
    otp[n_t] = tiles;
    uint64_t voff = 0;
    for (uint32_t v = 0; v < n_v; ++v) {
        PlanVec p;
        p.len2 = new_width[vecs[v].group];
        p.out_off = voff;
        p.pad = 0;
        pv[v] = p;
        voff += p.len2;
    }
    uint32_t status = 0;
    if (off > cap_w || voff > cap_v) status |= 1u;
    for (uint32_t g = 0; g < n_g; ++g)
        if (new_width[g] == 0) status |= 2u;
    hdr->elems_w = off;
    hdr->elems_v = voff;
    hdr->total_tiles = tiles;
    hdr->status = status;
}

// One block per tile of TILE consecutive elements of one rebuilt tensor.  Element
// (o', c', k) of the output comes from (keep_out[o'], keep_in[c'], k) of the source,
// where k runs over the kk = kh * kw * in_mult elements of one (filter, channel) pair.
__global__ __launch_bounds__(BLOCK) void gather_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups, uint32_t n_t,
    const PlanTensor* __restrict__ pt, const uint32_t* __restrict__ otp,
    const PlanHeader* __restrict__ hdr, const float* __restrict__ w,
    const uint32_t* __restrict__ keep, float* __restrict__ w_out) {
    if (hdr->status & 1u) return;
    const uint32_t tile = blockIdx.x;
    if (tile >= hdr->total_tiles) return;
    const uint32_t t = find_tensor(otp, n_t, tile);
    const DevTensor T = tens[t];
    const PlanTensor P = pt[t];
    const uint32_t e0 = (tile - otp[t]) * TILE;
    const uint32_t n = min(TILE, P.numel2 - e0);
    const uint32_t* keep_o = keep + groups[T.out_group].off;
    const uint32_t* keep_i = keep + groups[T.in_group].off;
    const uint32_t row2 = P.c2 * T.kk;
    const float* src = w + T.offset;
    float* dst = w_out + P.out_off + e0;
    for (uint32_t j = threadIdx.x; j < n; j += BLOCK) {
        const uint32_t idx = e0 + j;
        const uint32_t o2 = idx / row2;
        const uint32_t rem = idx - o2 * row2;
        const uint32_t c2 = rem / T.kk;
        const uint32_t k = rem - c2 * T.kk;
        const uint64_t s = ((uint64_t)keep_o[o2] * T.cin + keep_i[c2]) * T.kk + k;
        dst[j] = src[s];
    }
}

// One block per vector: v'[j] = v[keep[j]].
__global__ __launch_bounds__(BLOCK) void gather_vec_kernel(
    const DevVec* __restrict__ vecs, const DevGroup* __restrict__ groups,
    const PlanVec* __restrict__ pv, const PlanHeader* __restrict__ hdr,
    const float* __restrict__ v, const uint32_t* __restrict__ keep,
    float* __restrict__ v_out) {
    if (hdr->status & 1u) return;
    const DevVec V = vecs[blockIdx.x];
    const PlanVec P = pv[blockIdx.x];
    const uint32_t* kp = keep + groups[V.group].off;
    for (uint32_t j = threadIdx.x; j < P.len2; j += BLOCK)
        v_out[P.out_off + j] = v[V.offset + kp[j]];
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
                      uint32_t* d_keep, uint32_t* d_new_width) {
    const auto& b = m->b;
    ProfileScope p(ctx, K_PROPAGATE);
    propagate_kernel<<<(uint32_t)m->g.size(), BLOCK, 0, ctx->stream>>>(
        b.groups, b.producers, b.tens, d_out_alive, flags, d_group_alive, d_index_map, d_keep,
        d_new_width);
}

void launch_compact(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                    const float* d_vecs, const uint32_t* d_keep,
                    const uint32_t* d_new_width, float* d_w_out, uint64_t cap_w,
                    float* d_vecs_out, uint64_t cap_v) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size(), n_v = (uint32_t)m->v.size();
    {
        ProfileScope p(ctx, K_PLAN);
        plan_kernel<<<1, BLOCK, 0, ctx->stream>>>(b.tens, n_t, b.vecs, n_v, b.groups,
                                                  (uint32_t)m->g.size(), d_new_width, cap_w,
                                                  cap_v, b.plan_t, b.plan_v, b.out_tile_prefix,
                                                  b.plan_h);
    }
    {
        // worst-case grid (nothing removed); blocks past the real tile count exit at once
        ProfileScope p(ctx, K_GATHER);
        gather_kernel<<<m->n_tiles, BLOCK, 0, ctx->stream>>>(
            b.tens, b.groups, n_t, b.plan_t, b.out_tile_prefix, b.plan_h, d_w, d_keep, d_w_out);
    }
    if (n_v) {
        ProfileScope p(ctx, K_GATHER_VEC);
        gather_vec_kernel<<<n_v, BLOCK, 0, ctx->stream>>>(b.vecs, b.groups, b.plan_v, b.plan_h,
                                                          d_vecs, d_keep, d_vecs_out);
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
