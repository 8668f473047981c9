// K variants of a portfolio in one launch per step: the dense arena is read once and
// every variant's sparse arena and mask are written from it (Sec. III-C: a portfolio
// ranks and masks the same weights at growing sparsity; Sec. III-D Module 4: all layers
// pruned by one operation).
//
// The variants' kept sets are nested - a weight kept at a cut is kept at every smaller
// cut - so the zero-kernel / zero-channel analysis of Module 2 needs one number per
// filter and per input feature: its LEVEL, the largest count of variants that keep one
// of its non-zero weights.  A filter is alive in the variant holding the p-th smallest cut
// iff its level exceeds p.  Levels are maxima, so they are order-independent.
#include <algorithm>

#include "dev_common.h"

namespace shifter {

typedef uint32_t uint4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // dword-aligned

// pos[k] = number of variants whose cut is smaller than variant k's (ties by index).
__device__ __forceinline__ void load_cuts(const shifter_threshold* __restrict__ thr, uint32_t k_var,
                                          uint64_t* s_cut, uint32_t* s_pos) {
    if (threadIdx.x < k_var) s_cut[threadIdx.x] = thr[threadIdx.x].cut;
    __syncthreads();
    if (threadIdx.x < k_var) {
        const uint64_t mine = s_cut[threadIdx.x];
        uint32_t p = 0;
        for (uint32_t j = 0; j < k_var; ++j) {
            const uint64_t c = s_cut[j];
            p += (c < mine || (c == mine && j < threadIdx.x)) ? 1u : 0u;
        }
        s_pos[threadIdx.x] = p;
    }
    __syncthreads();
}

__global__ __launch_bounds__(BLOCK) void zero_u32_kernel(uint32_t* a, uint64_t n) {
    const uint64_t i = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (i < n) a[i] = 0;
}

template <bool NT>
__global__ __launch_bounds__(BLOCK) void mask_scan_batch_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix, uint32_t n_t,
    const float* __restrict__ w, const shifter_threshold* __restrict__ thr, uint32_t k_var,
    float* __restrict__ w_out, uint64_t w_stride, uint8_t* __restrict__ mask,
    uint64_t mask_stride, uint32_t* out_level, uint32_t* in_level) {
    __shared__ uint32_t rowmax[TILE + 16];
    __shared__ uint32_t colmax[TILE + 16];
    __shared__ uint64_t s_cut[MAXK];
    __shared__ uint32_t s_pos[MAXK];
    __shared__ __align__(16) uint32_t s_xm[TILE / 4];   // mask words of the tile, per wavefront

    const uint32_t tile = blockIdx.x;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    const DevTensor T = tens[t];
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const bool ranked = T.prunable != 0;
    const uint32_t g0 = (uint32_t)(T.gbase + e0);
    const uint32_t c0 = e0 % T.khw, r0 = e0 % T.row_len;
    const uint32_t nrows = (r0 + n - 1) / T.row_len + 1;
    const uint32_t ncols = (c0 + n - 1) / T.khw + 1;
    for (uint32_t s = threadIdx.x; s < nrows; s += BLOCK) rowmax[s] = 0;
    for (uint32_t s = threadIdx.x; s < ncols; s += BLOCK) colmax[s] = 0;
    load_cuts(thr, k_var, s_cut, s_pos);   // contains the barriers

    const float* src = w + T.offset + e0;
    const bool want_mask = ranked && mask != nullptr;

    // level of one weight = number of variants that keep it; marks its filter and kernel
    auto mark = [&](uint32_t j, uint32_t bits, uint32_t level) {
        if (level && (bits & 0x7fffffffu)) {
            atomicMax(&rowmax[div_small(r0 + j, T.row_len, T.magic_row)], level);
            atomicMax(&colmax[div_small(c0 + j, T.khw, T.magic_khw)], level);
        }
    };

    // w_out == nullptr: the sparse arenas are not wanted (the rebuild can mask the dense
    // arena on the way), only masks and levels are produced
    const bool vec_ok = n == TILE && (T.offset & 3u) == 0 && (!w_out || (w_stride & 3u) == 0) &&
                        (!want_mask || ((T.gbase & 3u) == 0 && (mask_stride & 3u) == 0));
    if (vec_ok) {
        // wavefront w owns the w-th quarter of the tile: quad 256 w + 64 u + lane in step u,
        // so every load and store covers 1 KB and the wavefront's mask bytes are one
        // contiguous KB - written with one 16-byte store per lane after a wavefront-local
        // exchange through LDS (four 4-byte stores cost as much issue time as four
        // 16-byte ones)
        constexpr uint32_t U = TILE / BLOCK / 4;
        const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
        const uint32_t q0 = wid * (64u * U) + lane;      // quad of step 0
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
        uint4 v[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) v[u] = load_u4<NT>(s4 + q0 + 64u * u);
        uint32_t lvl[U][4];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) lvl[u][0] = lvl[u][1] = lvl[u][2] = lvl[u][3] = 0;
        uint32_t* xm = s_xm + wid * (64u * U);
        for (uint32_t k = 0; k < k_var; ++k) {
            const uint64_t cut = ranked ? s_cut[k] : 0;
            float* dst = w_out + (uint64_t)k * w_stride + T.offset + e0;
            uint8_t* mdst = want_mask ? mask + (uint64_t)k * mask_stride + T.gbase + e0 : nullptr;
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t j = (q0 + 64u * u) * 4;
                const uint32_t b[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
                uint32_t o[4], keep[4];
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    const uint64_t comp = ((uint64_t)(b[q] & 0x7fffffffu) << 32) | (g0 + j + q);
                    keep[q] = comp < cut ? 0u : 1u;
                    o[q] = keep[q] ? b[q] : 0u;
                    lvl[u][q] += keep[q];
                }
                if (w_out)
                    store_u4<NT>(reinterpret_cast<uint4*>(dst) + q0 + 64u * u,
                                 make_uint4(o[0], o[1], o[2], o[3]));
                if (mdst) xm[64u * u + lane] = keep[0] | (keep[1] << 8) | (keep[2] << 16) | (keep[3] << 24);
            }
            if (mdst) {
                // lanes exchange within their own wavefront only: order the LDS accesses
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const uint4 mm = *reinterpret_cast<const uint4*>(xm + 4u * lane);
                uint4_a4 out;
                out.x = mm.x; out.y = mm.y; out.z = mm.z; out.w = mm.w;
                *reinterpret_cast<uint4_a4*>(mdst + wid * (256u * U) + 16u * lane) = out;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = (q0 + 64u * u) * 4;
            mark(j, v[u].x, lvl[u][0]);
            mark(j + 1, v[u].y, lvl[u][1]);
            mark(j + 2, v[u].z, lvl[u][2]);
            mark(j + 3, v[u].w, lvl[u][3]);
        }
    } else {
        for (uint32_t j = threadIdx.x; j < n; j += BLOCK) {
            const uint32_t bits = __float_as_uint(src[j]);
            const uint64_t comp = ((uint64_t)(bits & 0x7fffffffu) << 32) | (g0 + j);
            uint32_t level = 0;
            for (uint32_t k = 0; k < k_var; ++k) {
                const bool removed = ranked && comp < s_cut[k];
                level += removed ? 0u : 1u;
                if (w_out)
                    w_out[(uint64_t)k * w_stride + T.offset + e0 + j] = removed ? 0.0f : __uint_as_float(bits);
                if (want_mask) mask[(uint64_t)k * mask_stride + T.gbase + e0 + j] = removed ? 0 : 1;
            }
            mark(j, bits, level);
        }
    }
    __syncthreads();
    const uint32_t row_first = e0 / T.row_len;
    for (uint32_t s = threadIdx.x; s < nrows; s += BLOCK) {
        const uint32_t l = rowmax[s];
        if (l) {
            uint32_t* f = out_level + T.out_flag_off + row_first + s;
            if (*f < l) atomicMax(f, l);
        }
    }
    const uint32_t b = (e0 / T.khw) % T.in_ch;
    for (uint32_t s = threadIdx.x; s < ncols; s += BLOCK) {
        const uint32_t l = colmax[s];
        if (l) {
            uint32_t* f = in_level + T.in_flag_off + mod_small(b + s, T.in_ch, T.magic_in);
            if (*f < l) atomicMax(f, l);
        }
    }
}

// alive[k][i] = level[i] > pos[k], for the out and the in flags of every variant.
__global__ __launch_bounds__(BLOCK) void expand_levels_kernel(
    const shifter_threshold* __restrict__ thr, uint32_t k_var,
    const uint32_t* __restrict__ out_level, uint64_t n_out, const uint32_t* __restrict__ in_level,
    uint64_t n_in, uint8_t* __restrict__ out_alive, uint8_t* __restrict__ in_alive) {
    __shared__ uint64_t s_cut[MAXK];
    __shared__ uint32_t s_pos[MAXK];
    load_cuts(thr, k_var, s_cut, s_pos);
    const uint64_t i = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    const uint32_t k = blockIdx.y;
    if (i < n_out) out_alive[(uint64_t)k * n_out + i] = out_level[i] > s_pos[k] ? 1 : 0;
    if (i < n_in && in_alive) in_alive[(uint64_t)k * n_in + i] = in_level[i] > s_pos[k] ? 1 : 0;
}

void launch_zero_levels(shifter_ctx* ctx, const shifter_model* m) {
    const uint64_t n = m->info.sum_out_ch + m->info.sum_in_ch;
    ProfileScope p(ctx, K_ZERO_FLAGS);
    zero_u32_kernel<<<(uint32_t)((std::max<uint64_t>(n, 1) + BLOCK - 1) / BLOCK), BLOCK, 0, ctx->stream>>>(
        m->b.levels, n);
}

void launch_expand_levels(shifter_ctx* ctx, const shifter_model* m, const shifter_threshold* d_thr,
                          uint32_t k_var, uint8_t* d_out_alive, uint8_t* d_in_alive) {
    const uint64_t n_out = m->info.sum_out_ch, n_in = m->info.sum_in_ch;
    ProfileScope p(ctx, K_EXPAND_LEVELS);
    const uint64_t mx = std::max<uint64_t>(n_out > n_in ? n_out : n_in, 1);
    expand_levels_kernel<<<dim3((uint32_t)((mx + BLOCK - 1) / BLOCK), k_var), BLOCK, 0, ctx->stream>>>(
        d_thr, k_var, m->b.levels, n_out, m->b.levels + n_out, n_in, d_out_alive, d_in_alive);
}

void launch_mask_scan_batch(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                            const shifter_threshold* d_thr, uint32_t k_var, float* d_w_out,
                            uint64_t w_stride, uint8_t* d_mask, uint64_t mask_stride,
                            uint8_t* d_out_alive, uint8_t* d_in_alive) {
    launch_zero_levels(ctx, m);
    launch_mask_scan_batch_core(ctx, m, d_w, d_thr, k_var, d_w_out, w_stride, d_mask, mask_stride);
    launch_expand_levels(ctx, m, d_thr, k_var, d_out_alive, d_in_alive);
}

void launch_mask_scan_batch_core(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                                 const shifter_threshold* d_thr, uint32_t k_var, float* d_w_out,
                                 uint64_t w_stride, uint8_t* d_mask, uint64_t mask_stride) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size();
    const uint64_t n_out = m->info.sum_out_ch;
    hipStream_t s = ctx->stream;
    {
        ProfileScope p(ctx, K_MASK_SCAN_BATCH);
        // measured: with ten output streams per block the non-temporal hint costs about
        // 6 % on an arena far larger than the last-level cache (4.9 vs 5.2 TB/s); on an
        // arena that fits the cache it keeps the outputs from evicting what the rebuild
        // reads next and the whole step is faster with it
        const bool nt = m->info.w_extent * 4 <= (192ull << 20);
        auto k = nt ? mask_scan_batch_kernel<true> : mask_scan_batch_kernel<false>;
        k<<<m->n_tiles, BLOCK, 0, s>>>(b.tens, b.tile_prefix, n_t, d_w, d_thr, k_var, d_w_out,
                                       w_stride, d_mask, mask_stride, b.levels, b.levels + n_out);
    }
}

}  // namespace shifter
