// Threshold-and-mask pass (the sparse model of Sec. II-A / Sec. III-C) fused with the
// zero-kernel / zero-channel analysis of Module 2 (Sec. III-D), and the same analysis
// as a stand-alone pass.
//
// One block per tile of TILE consecutive elements of one tensor.  A weight is removed
// iff its 64-bit composite (magnitude key << 32 | global index) is below the cut of the
// threshold record: one integer compare, no tie path.  The scan marks, in LDS byte
// flags indexed relative to the tile's first filter and first kernel, every filter and
// every (filter, input feature) kernel that holds a surviving non-zero; the flags are
// then folded into the global out_alive / in_alive bytes (writes of the constant 1, so
// no atomics are needed and the result does not depend on scheduling).
#include "dev_common.h"

namespace shifter {

__global__ __launch_bounds__(BLOCK) void zero_flags_kernel(uint8_t* a, uint64_t na,
                                                           uint8_t* b, uint64_t nb) {
    const uint64_t i = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (i < na) a[i] = 0;
    if (i < nb) b[i] = 0;
}

template <bool DO_MASK, bool DO_SCAN, bool NT>
__global__ __launch_bounds__(BLOCK) void mask_scan_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    uint32_t n_t, const float* w, const shifter_threshold* __restrict__ thr, float* w_out,
    uint8_t* __restrict__ mask, uint8_t* out_alive, uint8_t* in_alive) {
    __shared__ uint8_t rowf[DO_SCAN ? TILE + 16 : 16];
    __shared__ uint8_t colf[DO_SCAN ? TILE + 16 : 16];

    const uint32_t tile = blockIdx.x;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    const DevTensor T = tens[t];
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const bool ranked = DO_MASK && T.prunable;
    const uint64_t cut = ranked ? thr->cut : 0;
    const uint32_t g0 = (uint32_t)(T.gbase + e0);   // N < 2^32: the index fits 32 bits
    const uint32_t c0 = e0 % T.khw, r0 = e0 % T.row_len;
    const uint32_t nrows = (r0 + n - 1) / T.row_len + 1;
    const uint32_t ncols = (c0 + n - 1) / T.khw + 1;

    if (DO_SCAN) {
        for (uint32_t s = threadIdx.x; s < nrows; s += BLOCK) rowf[s] = 0;
        for (uint32_t s = threadIdx.x; s < ncols; s += BLOCK) colf[s] = 0;
        __syncthreads();
    }

    const float* src = w + T.offset + e0;
    float* dst = DO_MASK ? w_out + T.offset + e0 : nullptr;
    uint8_t* mdst = (ranked && mask) ? mask + T.gbase + e0 : nullptr;

    // returns the bits to store; marks the scan flags
    auto one = [&](uint32_t j, uint32_t bits, uint32_t& keep) -> uint32_t {
        const uint32_t key = bits & 0x7fffffffu;
        const bool removed = (((uint64_t)key << 32) | (uint64_t)(g0 + j)) < cut;
        keep = removed ? 0u : 1u;
        const uint32_t out = removed ? 0u : bits;
        if (DO_SCAN && !removed && key != 0) {
            const uint32_t rs = div_small(r0 + j, T.row_len, T.magic_row);
            const uint32_t cs = div_small(c0 + j, T.khw, T.magic_khw);
            rowf[rs] = 1;
            colf[cs] = 1;
        }
        return out;
    };

    const bool vec_ok = n == TILE && (T.offset & 3u) == 0 && (!mdst || (T.gbase & 3u) == 0);
    if (vec_ok) {
        constexpr uint32_t U = TILE / BLOCK / 4;
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
        uint4 v[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) v[u] = load_u4<NT>(s4 + threadIdx.x + BLOCK * u);
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = (threadIdx.x + BLOCK * u) * 4;
            uint32_t k0, k1, k2, k3;
            uint4 o;
            o.x = one(j, v[u].x, k0);
            o.y = one(j + 1, v[u].y, k1);
            o.z = one(j + 2, v[u].z, k2);
            o.w = one(j + 3, v[u].w, k3);
            if (DO_MASK) {
                store_u4<NT>(reinterpret_cast<uint4*>(dst) + threadIdx.x + BLOCK * u, o);
                if (mdst)
                    store_u1<NT>(reinterpret_cast<uint32_t*>(mdst) + threadIdx.x + BLOCK * u,
                                 k0 | (k1 << 8) | (k2 << 16) | (k3 << 24));
            }
        }
    } else {
        for (uint32_t j = threadIdx.x; j < n; j += BLOCK) {
            uint32_t k;
            const uint32_t o = one(j, __float_as_uint(src[j]), k);
            if (DO_MASK) {
                dst[j] = __uint_as_float(o);
                if (mdst) mdst[j] = (uint8_t)k;
            }
        }
    }

    if (DO_SCAN) {
        __syncthreads();
        const uint32_t row_first = e0 / T.row_len;
        for (uint32_t s = threadIdx.x; s < nrows; s += BLOCK) {
            if (rowf[s]) {
                uint8_t* f = out_alive + T.out_flag_off + row_first + s;
                if (*f == 0) *f = 1;
            }
        }
        const uint32_t b = (e0 / T.khw) % T.in_ch;   // input feature of the tile's first kernel
        for (uint32_t s = threadIdx.x; s < ncols; s += BLOCK) {
            if (colf[s]) {
                const uint32_t i = mod_small(b + s, T.in_ch, T.magic_in);
                uint8_t* f = in_alive + T.in_flag_off + i;
                if (*f == 0) *f = 1;
            }
        }
    }
}

static void zero_flags(shifter_ctx* ctx, const shifter_model* m, uint8_t* d_out_alive,
                       uint8_t* d_in_alive) {
    const uint64_t na = m->info.sum_out_ch, nb = m->info.sum_in_ch;
    const uint64_t mx = na > nb ? na : nb;
    ProfileScope p(ctx, K_ZERO_FLAGS);
    zero_flags_kernel<<<(uint32_t)((mx + BLOCK - 1) / BLOCK), BLOCK, 0, ctx->stream>>>(
        d_out_alive, na, d_in_alive, nb);
}

// Arenas beyond this size cannot stay in the 256 MB last-level cache between passes:
// stream them with the non-temporal hint.
static bool streaming(const shifter_model* m) { return m->info.w_extent * 4 > (192ull << 20); }

void launch_mask_scan(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                      const shifter_threshold* d_thr, float* d_w_out, uint8_t* d_mask,
                      uint8_t* d_out_alive, uint8_t* d_in_alive) {
    const auto& b = m->b;
    const uint32_t n_t = (uint32_t)m->t.size();
    const bool nt = streaming(m);
    if (d_out_alive) {
        zero_flags(ctx, m, d_out_alive, d_in_alive);
        ProfileScope p(ctx, K_MASK_SCAN);
        auto k = nt ? mask_scan_kernel<true, true, true> : mask_scan_kernel<true, true, false>;
        k<<<m->n_tiles, BLOCK, 0, ctx->stream>>>(b.tens, b.tile_prefix, n_t, d_w, d_thr, d_w_out,
                                                 d_mask, d_out_alive, d_in_alive);
    } else {
        ProfileScope p(ctx, K_MASK_SCAN);
        auto k = nt ? mask_scan_kernel<true, false, true> : mask_scan_kernel<true, false, false>;
        k<<<m->n_tiles, BLOCK, 0, ctx->stream>>>(b.tens, b.tile_prefix, n_t, d_w, d_thr, d_w_out,
                                                 d_mask, nullptr, nullptr);
    }
}

void launch_scan(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                 uint8_t* d_out_alive, uint8_t* d_in_alive) {
    const auto& b = m->b;
    zero_flags(ctx, m, d_out_alive, d_in_alive);
    ProfileScope p(ctx, K_SCAN);
    auto k = streaming(m) ? mask_scan_kernel<false, true, true> : mask_scan_kernel<false, true, false>;
    k<<<m->n_tiles, BLOCK, 0, ctx->stream>>>(b.tens, b.tile_prefix, (uint32_t)m->t.size(), d_w,
                                             nullptr, nullptr, nullptr, d_out_alive, d_in_alive);
}

}  // namespace shifter
