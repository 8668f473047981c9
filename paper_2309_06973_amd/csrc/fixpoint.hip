// Liveness fixpoint of the prune plan on the kernel-level zero index (an extension beyond
// Algorithm 1's single pass, on Module 2's index of zero kernels, Sec. III-D): a channel
// stays only while (produced) some filter writing it has a non-zero kernel on an alive
// input feature and (read) some alive filter reads it through a non-zero kernel.  The
// rules are applied to all channels at once, round after round, until a round removes
// nothing; removal only makes more channels fail, so the result does not depend on the
// order of removal.
#include <algorithm>

#include "dev_common.h"

namespace shifter {

constexpr uint32_t FIX_ROWS = 16;     // filters per tile of the kernel index
constexpr uint32_t FIX_COLS = 1024;   // kernels of a filter per tile (4 per thread)

__global__ __launch_bounds__(BLOCK) void fill_u8_kernel(uint8_t* a, uint64_t n, uint8_t v) {
    const uint64_t i = ((uint64_t)blockIdx.x * BLOCK + threadIdx.x) * 16u;
    if (i + 16u <= n && (reinterpret_cast<uintptr_t>(a + i) & 15u) == 0) {
        const uint32_t x = v * 0x01010101u;
        *reinterpret_cast<uint4*>(a + i) = make_uint4(x, x, x, x);
    } else {
        for (uint64_t j = i; j < n && j < i + 16u; ++j) a[j] = v;
    }
}

// Module 2's kernel-level index: nz[koff_t + o * in_ch + i] = 1 iff the kh x kw kernel of
// filter o and input feature i of tensor t holds a non-zero.  One tile of 4096 weights per
// block; a kernel that straddles two tiles is set by either (the array starts zeroed).
__global__ __launch_bounds__(BLOCK) void kernel_scan_kernel(
    const DevTensor* __restrict__ tens, const uint32_t* __restrict__ tile_prefix, uint32_t n_t,
    const uint64_t* __restrict__ kernel_off, const float* __restrict__ w,
    uint8_t* __restrict__ nz) {
    __shared__ uint8_t flag[TILE + 16];
    const uint32_t tile = blockIdx.x;
    const uint32_t t = find_tensor(tile_prefix, n_t, tile);
    const DevTensor T = tens[t];
    const uint32_t e0 = (tile - tile_prefix[t]) * TILE;
    const uint32_t n = min(TILE, T.numel - e0);
    const uint32_t c0 = e0 % T.khw;                     // offset inside the first kernel
    const uint32_t n_k = (c0 + n - 1) / T.khw + 1;      // kernels touched by the tile
    for (uint32_t s = threadIdx.x; s < n_k; s += BLOCK) flag[s] = 0;
    __syncthreads();
    const float* src = w + T.offset + e0;
    auto mark = [&](uint32_t j, uint32_t bits) {
        if (bits & 0x7fffffffu) flag[div_small(c0 + j, T.khw, T.magic_khw)] = 1;
    };
    if (n == TILE && (T.offset & 3u) == 0) {
        constexpr uint32_t U = TILE / BLOCK / 4;
        const uint4* s4 = reinterpret_cast<const uint4*>(src);
        uint4 v[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) v[u] = load_u4<false>(s4 + threadIdx.x + BLOCK * u);
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = (threadIdx.x + BLOCK * u) * 4;
            mark(j, v[u].x); mark(j + 1, v[u].y); mark(j + 2, v[u].z); mark(j + 3, v[u].w);
        }
    } else {
        for (uint32_t j = threadIdx.x; j < n; j += BLOCK) mark(j, __float_as_uint(src[j]));
    }
    __syncthreads();
    uint8_t* dst = nz + kernel_off[t] + e0 / T.khw;
    for (uint32_t s = threadIdx.x; s < n_k; s += BLOCK)
        if (flag[s]) dst[s] = 1;
}

// The rounds of a call are enqueued one behind the other with no wait between them:
// removed[j] counts what round j of the batch took away (removed[0] stands for the round
// before the batch and starts at 1), and the kernels of round j return at once when
// removed[j - 1] is 0, which is then true of every later round too.
//
// One round, first half: a tile of FIX_ROWS filters x FIX_COLS kernels of one tensor's
// index.  produced[t][o] is set if filter o has a non-zero kernel on an alive feature;
// read[t][i] is set if feature i has a non-zero kernel in a filter whose channel is alive.
// Both arrays are zero when the round starts and only ever get ones.
__global__ __launch_bounds__(BLOCK) void fix_tile_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups, uint32_t n_t,
    const uint32_t* __restrict__ fix_prefix, const uint64_t* __restrict__ kernel_off,
    const uint8_t* __restrict__ nz, const uint8_t* __restrict__ alive,
    uint8_t* __restrict__ produced, uint8_t* __restrict__ read,
    const uint32_t* __restrict__ removed_before) {
    if (*removed_before == 0) return;     // the round before removed nothing: settled
    const uint32_t t = find_tensor(fix_prefix, n_t, blockIdx.x);
    const DevTensor T = tens[t];
    const uint32_t chunks = (T.in_ch + FIX_COLS - 1) / FIX_COLS;
    const uint32_t local = blockIdx.x - fix_prefix[t];
    const uint32_t band = local / chunks, chunk = local - band * chunks;
    const uint32_t o0 = band * FIX_ROWS, o1 = min(T.out_ch, o0 + FIX_ROWS);
    const uint32_t i0 = chunk * FIX_COLS + threadIdx.x * 4u;
    const uint32_t in_mult = T.in_ch / T.cin;
    const uint8_t* a_in = alive + groups[T.in_group].off;
    const uint8_t* a_out = alive + groups[T.out_group].off;
    uint32_t in_ok = 0;       // byte q: feature i0 + q exists and its channel is alive
    for (uint32_t q = 0; q < 4; ++q)
        if (i0 + q < T.in_ch && a_in[(i0 + q) / in_mult]) in_ok |= 0xffu << (8 * q);
    const uint8_t* base = nz + kernel_off[t];
    uint32_t col_hit = 0;
    // the FIX_ROWS loads of a thread go out together
    uint32_t v[FIX_ROWS];
    const bool whole = i0 + 3 < T.in_ch;
#pragma unroll
    for (uint32_t r = 0; r < FIX_ROWS; ++r) {
        const uint32_t o = min(o0 + r, o1 - 1);
        const uint8_t* row = base + (uint64_t)o * T.in_ch + i0;
        v[r] = 0;
        if (whole && (reinterpret_cast<uintptr_t>(row) & 3u) == 0) {
            v[r] = *reinterpret_cast<const uint32_t*>(row);
        } else {
            for (uint32_t q = 0; q < 4; ++q)
                if (i0 + q < T.in_ch) v[r] |= (uint32_t)row[q] << (8 * q);
        }
    }
#pragma unroll
    for (uint32_t r = 0; r < FIX_ROWS; ++r) {
        const uint32_t o = o0 + r;
        if (o >= o1) break;
        if (a_out[o]) col_hit |= v[r];
        if (__ballot((v[r] & in_ok) != 0) != 0 && (threadIdx.x & 63u) == 0)
            produced[T.out_flag_off + o] = 1;
    }
    for (uint32_t q = 0; q < 4; ++q)
        if ((col_hit >> (8 * q)) & 0xffu) read[T.in_flag_off + i0 + q] = 1;
}

// One round, second half, one block per group: alive[c] &= produced by some producer and
// read by some consumer (pinned and frozen groups stay whole).  The entries this block
// reads are its own; it zeroes them for the next round.  Counts the channels it removes.
__global__ __launch_bounds__(BLOCK) void fix_update_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups,
    const uint32_t* __restrict__ producers, const uint32_t* __restrict__ cons_prefix,
    const uint32_t* __restrict__ consumers, uint32_t flags, uint8_t* __restrict__ alive,
    uint8_t* __restrict__ produced, uint8_t* __restrict__ read,
    const uint32_t* __restrict__ removed_before, uint32_t* __restrict__ removed) {
    if (*removed_before == 0) return;
    const DevGroup G = groups[blockIdx.x];
    const uint32_t n_prod = G.prod_end - G.prod_begin;
    const bool frozen = G.pinned || ((flags & SHIFTER_PAPER_FREEZE_RESIDUAL) && n_prod > 1);
    uint32_t gone = 0;
    for (uint32_t c = threadIdx.x; c < G.width; c += BLOCK) {
        uint32_t p = 0, r = 0;
        for (uint32_t k = G.prod_begin; k < G.prod_end; ++k) {
            uint8_t* f = produced + tens[producers[k]].out_flag_off + c;
            p |= *f;
            *f = 0;
        }
        for (uint32_t k = cons_prefix[blockIdx.x]; k < cons_prefix[blockIdx.x + 1]; ++k) {
            const DevTensor& T = tens[consumers[k]];
            const uint32_t m = T.in_ch / T.cin;
            for (uint32_t q = 0; q < m; ++q) {
                uint8_t* f = read + T.in_flag_off + c * m + q;
                r |= *f;
                *f = 0;
            }
        }
        if (!frozen && alive[G.off + c] && !(p && r)) {
            alive[G.off + c] = 0;
            ++gone;
        }
    }
    if (gone) atomicAdd(removed, gone);
}

// Start of a call, one launch: all channels alive, no flags, removed[0] = 1 so that the
// first round runs.  Blocks [0, ba) fill alive, [ba, bp) produced, [bp, br) read, each 16
// bytes per thread; the last block sets the state words.
__global__ __launch_bounds__(BLOCK) void fix_begin_kernel(uint8_t* alive, uint64_t n_alive, uint8_t* produced,
                                                         uint64_t n_prod, uint8_t* read, uint64_t n_read,
                                                         uint32_t ba, uint32_t bp, uint32_t br,
                                                         uint32_t* __restrict__ st) {
    uint32_t blk = blockIdx.x;
    if (blk >= br) {
        if (threadIdx.x < FIX_STATE_WORDS) st[threadIdx.x] = threadIdx.x == 0 ? 1u : 0u;
        return;
    }
    uint8_t* a = alive;
    uint64_t n = n_alive;
    uint8_t v = 1;
    if (blk >= bp) { a = read; n = n_read; v = 0; blk -= bp; }
    else if (blk >= ba) { a = produced; n = n_prod; v = 0; blk -= ba; }
    const uint64_t i = ((uint64_t)blk * BLOCK + threadIdx.x) * 16u;
    if (i + 16u <= n && (reinterpret_cast<uintptr_t>(a + i) & 15u) == 0) {
        const uint32_t x = v * 0x01010101u;
        *reinterpret_cast<uint4*>(a + i) = make_uint4(x, x, x, x);
    } else {
        for (uint64_t j = i; j < n && j < i + 16u; ++j) a[j] = v;
    }
}

// End of a batch of FIX_BATCH rounds.  out_flags[t][o] = alive[out_group(t)][o]: the alive
// sets in the shape the planner's scan step takes, so that index maps and keep lists come
// from the same kernel as ever.  The first thread also closes the batch: it adds the rounds
// that ran to the total, carries removed[FIX_BATCH] to removed[0] for a batch that may
// follow, clears the other counters and writes (rounds, settled) to the pinned mirror.
__global__ __launch_bounds__(BLOCK) void fix_finish_kernel(
    const DevTensor* __restrict__ tens, const DevGroup* __restrict__ groups,
    const uint8_t* __restrict__ alive, uint8_t* __restrict__ out_flags, uint32_t* __restrict__ st,
    uint32_t* __restrict__ mirror) {
    if (blockIdx.x == gridDim.x - 1) {
        if (threadIdx.x == 0) {
            uint32_t ran = 0;
            for (uint32_t j = 1; j <= FIX_BATCH; ++j) ran += st[j - 1] != 0;
            const uint32_t last = st[FIX_BATCH];
            const uint32_t rounds = st[FIX_BATCH + 1] + ran;
            for (uint32_t j = 1; j <= FIX_BATCH; ++j) st[j] = 0;
            st[0] = last;
            st[FIX_BATCH + 1] = rounds;
            mirror[0] = rounds;
            mirror[1] = last == 0;
        }
        return;
    }
    const DevTensor& T = tens[blockIdx.x];
    const uint8_t* a = alive + groups[T.out_group].off;
    for (uint32_t o = threadIdx.x; o < T.out_ch; o += BLOCK) out_flags[T.out_flag_off + o] = a[o];
}

void launch_kernel_scan(shifter_ctx* ctx, const shifter_model* m, const float* d_w, uint8_t* d_nz) {
    const auto& b = m->b;
    hipStream_t s = ctx->stream;
    {
        ProfileScope p(ctx, K_ZERO_FLAGS);
        const uint64_t n = std::max<uint64_t>(m->sum_kernels, 1);
        fill_u8_kernel<<<(uint32_t)((n + BLOCK * 16 - 1) / (BLOCK * 16)), BLOCK, 0, s>>>(d_nz, n, 0);
    }
    if (m->n_tiles) {
        ProfileScope p(ctx, K_KERNEL_SCAN);
        kernel_scan_kernel<<<m->n_tiles, BLOCK, 0, s>>>(b.tens, b.tile_prefix, (uint32_t)m->t.size(),
                                                       b.kernel_off, d_w, d_nz);
    }
}

__global__ __launch_bounds__(BLOCK) void fix_widths_kernel(const uint32_t* __restrict__ w,
                                                          uint32_t* __restrict__ mirror, uint32_t n) {
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK) mirror[i] = w[i];
}

// The plan's widths into the pinned mirror the host reads after its wait.
void launch_fix_widths(shifter_ctx* ctx, const shifter_model* m, const uint32_t* d_new_width) {
    ProfileScope p(ctx, K_FIX_ROUND);
    fix_widths_kernel<<<1, BLOCK, 0, ctx->stream>>>(d_new_width, m->b.dev_width, (uint32_t)m->g.size());
}

void launch_fix_begin(shifter_ctx* ctx, const shifter_model* m) {
    const auto& b = m->b;
    ProfileScope p(ctx, K_ZERO_FLAGS);
    const uint64_t ng = m->info.sum_group_width, no = m->info.sum_out_ch, ni = m->info.sum_in_ch;
    auto blocks = [](uint64_t n) { return (uint32_t)((n + BLOCK * 16 - 1) / (BLOCK * 16)); };
    const uint32_t ba = blocks(ng), bp = ba + blocks(no), br = bp + blocks(ni);
    fix_begin_kernel<<<br + 1, BLOCK, 0, ctx->stream>>>(b.fix_alive, ng, b.fix_produced, no, b.fix_read, ni,
                                                        ba, bp, br, b.fix_removed);
}

// One batch: FIX_BATCH rounds back to back, then the kernel that closes it.
void launch_fix_batch(shifter_ctx* ctx, const shifter_model* m, const uint8_t* d_nz, uint32_t flags) {
    const auto& b = m->b;
    hipStream_t s = ctx->stream;
    ProfileScope p(ctx, K_FIX_ROUND);
    for (uint32_t j = 1; j <= FIX_BATCH; ++j) {
        if (m->fix_prefix.back())
            fix_tile_kernel<<<m->fix_prefix.back(), BLOCK, 0, s>>>(
                b.tens, b.groups, (uint32_t)m->t.size(), b.fix_prefix, b.kernel_off, d_nz, b.fix_alive,
                b.fix_produced, b.fix_read, b.fix_removed + j - 1);
        if (!m->g.empty())
            fix_update_kernel<<<(uint32_t)m->g.size(), BLOCK, 0, s>>>(
                b.tens, b.groups, b.producers, b.cons_prefix, b.consumers, flags, b.fix_alive,
                b.fix_produced, b.fix_read, b.fix_removed + j - 1, b.fix_removed + j);
    }
    fix_finish_kernel<<<(uint32_t)m->t.size() + 1, BLOCK, 0, s>>>(
        b.tens, b.groups, b.fix_alive, b.fix_out_flags, b.fix_removed,
        reinterpret_cast<uint32_t*>(b.dev_multi_status) + FIX_MIRROR_WORD);
}

}  // namespace shifter
