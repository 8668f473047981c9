// Conv + BatchNorm fold (Sec. III-D, Module 1): every filter o of a layer followed by a
// BatchNorm is scaled by s_o = gamma_o / sqrt(var_o + eps) and the layer gets the bias
// beta_o + (b_o - mean_o) * s_o, after which the BatchNorm vectors are not needed any
// more.  fp32 throughout: s_o is one correctly rounded add, square root and division, the
// weight one more multiplication, the bias one subtraction and one fused multiply-add.
// Streaming work: one read and one write of the weight arena.
#include "dev_common.h"

namespace shifter {

// Scale of every filter (1 for layers without a BatchNorm) and the folded biases.
// grid: (ceil(max out_ch / BLOCK), n_tensors).
__global__ __launch_bounds__(BLOCK) void fold_scale_kernel(
    const DevTensor* __restrict__ tens, const FoldTensor* __restrict__ fold,
    const float* __restrict__ vecs, float eps, float* __restrict__ scale,
    float* __restrict__ bias_out) {
    const uint32_t t = blockIdx.y;
    const uint32_t o = blockIdx.x * BLOCK + threadIdx.x;
    const DevTensor T = tens[t];
    if (o >= T.out_ch) return;
    const FoldTensor F = fold[t];
    float s = 1.0f;
    float b = F.bias >= 0 ? vecs[F.bias + o] : 0.0f;
    if (F.gamma >= 0) {
        s = vecs[F.gamma + o] / sqrtf(vecs[F.var + o] + eps);
        b = fmaf(b - vecs[F.mean + o], s, vecs[F.beta + o]);
    }
    scale[T.out_flag_off + o] = s;
    if (F.out_offset >= 0) bias_out[F.out_offset + o] = b;
}

// One tile of TILE weights per block: w_out = w * scale[filter of the weight].  The scales
// of the filters that the tile touches are staged in LDS first.  w_out may be w.
template <bool NT>
__global__ __launch_bounds__(BLOCK) void fold_apply_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix,
    const uint16_t* __restrict__ tile_tensor, const float* __restrict__ scale,
    const float* __restrict__ w, float* __restrict__ w_out) {
    __shared__ float s_scale[TILE + 1];
    const uint32_t tile = blockIdx.x;
    const uint32_t t = tile_tensor[tile];
    const DevTensor T = tens[t];
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const uint32_t r0 = e0 / T.row_len;
    const uint32_t c0 = e0 - r0 * T.row_len;            // offset inside the first filter
    const uint32_t n_rows = (c0 + n - 1) / T.row_len + 1;
    const float* sc = scale + T.out_flag_off + r0;
    for (uint32_t r = threadIdx.x; r < n_rows; r += BLOCK) s_scale[r] = sc[r];
    const float* src = w + T.offset + e0;
    float* dst = w_out + T.offset + e0;
    if (n == TILE && (T.offset & 3u) == 0) {
        constexpr uint32_t U = TILE / BLOCK / 4;
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
        uint4* d4 = reinterpret_cast<uint4*>(dst);
        uint4 v[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) v[u] = load_u4<NT>(s4 + threadIdx.x + BLOCK * u);
        __syncthreads();
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = c0 + (threadIdx.x + BLOCK * u) * 4;
            auto mul = [&](uint32_t bits, uint32_t jj) {
                return __float_as_uint(__uint_as_float(bits) *
                                       s_scale[div_small(jj, T.row_len, T.magic_row)]);
            };
            const uint4 r = make_uint4(mul(v[u].x, j), mul(v[u].y, j + 1), mul(v[u].z, j + 2),
                                       mul(v[u].w, j + 3));
            store_u4<NT>(d4 + threadIdx.x + BLOCK * u, r);
        }
    } else {
        __syncthreads();
        for (uint32_t j = threadIdx.x; j < n; j += BLOCK)
            dst[j] = src[j] * s_scale[div_small(c0 + j, T.row_len, T.magic_row)];
    }
}

void launch_fold(shifter_ctx* ctx, const shifter_model* m, const float* d_w, const float* d_vecs,
                 float eps, float* d_w_out, float* d_bias_out) {
    const auto& b = m->b;
    const uint32_t n_t = m->info.n_tensors;
    if (n_t == 0) return;
    uint32_t max_out = 1;
    for (const auto& t : m->dt) max_out = std::max(max_out, t.out_ch);
    {
        ProfileScope ps(ctx, K_FOLD_SCALE);
        fold_scale_kernel<<<dim3((max_out + BLOCK - 1) / BLOCK, n_t), BLOCK, 0, ctx->stream>>>(
            b.tens, b.fold, d_vecs, eps, b.fold_scale, d_bias_out);
    }
    if (m->n_tiles == 0) return;
    ProfileScope ps(ctx, K_FOLD_APPLY);
    // arenas that fit the last-level cache are re-read by the steps that follow
    if (m->info.w_extent * 4 > (192ull << 20))
        fold_apply_kernel<true><<<m->n_tiles, BLOCK, 0, ctx->stream>>>(
            b.tens, b.tile_prefix, b.tile_tensor, b.fold_scale, d_w, d_w_out);
    else
        fold_apply_kernel<false><<<m->n_tiles, BLOCK, 0, ctx->stream>>>(
            b.tens, b.tile_prefix, b.tile_tensor, b.fold_scale, d_w, d_w_out);
}

}  // namespace shifter
