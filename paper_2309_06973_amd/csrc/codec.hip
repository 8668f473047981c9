// Portfolio codec (Sec. III-E, Modules 7 and 8): inactive models are kept as DEFLATE
// streams (RFC 1951) and inflated when they are to run.  The encoder is built for
// chunk-parallel work on both sides:
//   - chunks of 32768 bytes, each its own byte-aligned segment of the stream; inside a
//     chunk 64 sub-chunks of 512 bytes, one lane each;
//   - tokens: literals, and for a run of r >= 4 equal bytes inside a sub-chunk one literal
//     followed by distance-1 matches over the other r - 1 bytes (258 while more than 260
//     remain, then one piece, or (rest - 3, 3) when 259 or 260 remain);
//   - a sub-chunk whose tokens would take more than 8 * bytes + 48 bits is stored: a stored
//     block of its own; the others are coded with the fixed Huffman codes;
//   - a segment walks its sub-chunks: a coded one opens a fixed-Huffman block unless one is
//     open and appends its tokens, a stored one closes the open block and is a stored
//     block; at the end the open block is closed and an empty stored block pads to a byte
//     (and carries BFINAL in the last segment).  If that is not shorter than one stored
//     block with the whole chunk, the segment is that block;
//   - side information for the decoder: the byte offset of every segment, and per
//     sub-chunk its token bits, or 0xFFFF if stored (all 0: whole chunk in one block).
// Any inflater reads the stream; the decoder here reads this encoder's streams, one wave
// per chunk, one lane per sub-chunk.
#include <string>

#include "dev_common.h"

namespace shifter {

constexpr uint32_t CODEC_CHUNK = SHIFTER_CODEC_CHUNK;
constexpr uint32_t CODEC_SUB = SHIFTER_CODEC_SUB;
constexpr uint32_t CODEC_NSUB = CODEC_CHUNK / CODEC_SUB;      // 64: one wave
constexpr uint32_t CODEC_SUBW = CODEC_SUB / 4;                // dwords per sub-chunk
constexpr uint32_t CODEC_SLOT = CODEC_CHUNK + 8;              // bytes of a chunk's slot in the workspace
constexpr uint32_t CODEC_MARGIN = 48;                         // bits a stored sub-chunk must save
constexpr uint32_t CODEC_STORED = 0xFFFFu;                    // side information of a stored sub-chunk
constexpr uint32_t CODEC_MASKW = CODEC_SUB / 32 + 1;          // run-start mask words per lane, padded
static_assert(CODEC_NSUB == 64, "one lane per sub-chunk");

enum : uint32_t { CODEC_BAD_STREAM = 1u, CODEC_CAPACITY = 2u };

// Sub-chunk l, dword j of the chunk staged in LDS: every row is rotated by l 16-byte
// vectors, so that the lanes of a wave, each walking its own sub-chunk at the same pace,
// spread over the banks while a vector stays whole.
__device__ __forceinline__ uint32_t sub_word(uint32_t l, uint32_t j) {
    return l * CODEC_SUBW + ((j + 4u * l) & (CODEC_SUBW - 1));
}

// Fixed literal code of RFC 1951 section 3.2.6, bit-reversed so that it can be appended
// from the least significant bit; returns the number of bits.
__device__ __forceinline__ uint32_t literal_code(uint32_t v, uint32_t* code) {
    const bool nine = v >= 144u;                  // 0x30 + v in 8 bits, or 0x190 + (v - 144) in 9
    *code = __brev(nine ? 0x100u + v : 0x30u + v) >> (nine ? 23u : 24u);
    return nine ? 9u : 8u;
}

// A match of `len` (3..258) at distance 1: length code, extra bits, 5-bit distance code 0.
__device__ __forceinline__ uint32_t match_code(uint32_t len, uint32_t* code) {
    uint32_t idx, e = 0, extra = 0;
    if (len == 258u) {
        idx = 28u;
    } else if (len < 11u) {
        idx = len - 3u;
    } else {
        const uint32_t x = len - 3u;              // 8..254
        e = 29u - (uint32_t)__clz(x);             // floor(log2 x) - 2
        idx = 4u * e + 4u + ((x >> e) & 3u);
        extra = x & ((1u << e) - 1u);
    }
    uint32_t c, n;
    if (idx < 23u) { c = __brev(1u + idx) >> 25; n = 7u; }         // symbols 257..279
    else { c = __brev(0xC0u + (idx - 23u)) >> 24; n = 8u; }        // symbols 280..285
    *code = c | (extra << n);
    return n + e + 5u;
}

struct BitCounter {
    uint32_t bits = 0;
    __device__ __forceinline__ void put(uint32_t, uint32_t n) { bits += n; }
};

// Appends bits to the chunk's bit buffer in LDS, which starts zeroed: every dword is OR-ed
// in, so neighbouring lanes may share the dwords at the ends of their ranges.  At most 32
// bits per call.
struct BitWriter {
    uint32_t* buf;
    uint64_t acc;
    uint32_t cnt, widx;
    __device__ __forceinline__ BitWriter(uint32_t* b, uint32_t start_bit)
        : buf(b), acc(0), cnt(start_bit & 31u), widx(start_bit >> 5) {}
    __device__ __forceinline__ void put(uint32_t code, uint32_t n) {
        acc |= (uint64_t)code << cnt;
        cnt += n;
        if (cnt >= 32u) {
            atomicOr(&buf[widx], (uint32_t)acc);
            ++widx;
            acc >>= 32;
            cnt -= 32u;
        }
    }
    __device__ __forceinline__ void finish() {
        if (cnt) atomicOr(&buf[widx], (uint32_t)acc);
    }
};

// Bits of the distance-1 matches that cover the `rest` >= 3 bytes after a run's first byte.
template <class Sink>
__device__ __forceinline__ void put_matches(uint32_t rest, Sink& sink) {
    uint32_t code, nb;
    while (rest > 260u) {
        nb = match_code(258u, &code);
        sink.put(code, nb);
        rest -= 258u;
    }
    if (rest <= 258u) {
        nb = match_code(rest, &code);
        sink.put(code, nb);
    } else {
        nb = match_code(rest - 3u, &code);
        sink.put(code, nb);
        nb = match_code(3u, &code);
        sink.put(code, nb);
    }
}

// First set bit of the mask row `mk` at a position after p (the row ends with a set bit).
__device__ __forceinline__ uint32_t next_bit(const uint32_t* mk, uint32_t p) {
    uint32_t a = (p + 1u) >> 5;
    uint32_t mw = mk[a] & (~0u << ((p + 1u) & 31u));
    while (mw == 0u && a + 1u < CODEC_MASKW) mw = mk[++a];
    return mw ? a * 32u + (uint32_t)__ffs((int)mw) - 1u : CODEC_SUB;
}

// Tokens of sub-chunk `l` (n > 0 bytes).  mk: one bit per byte that is sent as a literal
// (run starts, and every byte of a run shorter than 4), plus a set bit at position n: the
// distance from a literal to the next one is 1, or the length of the run it starts.
template <class Sink>
__device__ __forceinline__ void encode_sub(const uint32_t* s_in, const uint32_t* mk, uint32_t l,
                                           uint32_t n, Sink& sink) {
    uint32_t p = 0;
    while (p < n) {
        const uint32_t q = next_bit(mk, p);
        const uint32_t b = (s_in[sub_word(l, p >> 2)] >> ((p & 3u) * 8u)) & 0xffu;
        uint32_t code;
        const uint32_t nb = literal_code(b, &code);
        sink.put(code, nb);
        if (q - p >= 4u) put_matches(q - p - 1u, sink);
        p = q;
    }
}

__device__ __forceinline__ uint32_t wave_excl_scan(uint32_t v, uint32_t lane, uint32_t* total) {
    uint32_t x = v;
    for (uint32_t d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    *total = __shfl(x, 63, 64);
    return x - v;
}

// Where every sub-chunk's part of a segment starts, from the side information (s_side:
// token bits, or CODEC_STORED) and the chunk's size.  start: bit position of the first bit
// this lane's sub-chunk is responsible for (a coded one: the block header if it opens a
// block, then its tokens; a stored one: the end-of-block of the block it closes, then its
// own header); in_block: whether a Huffman block is open at that point.  tail_*: the same
// for what follows the last sub-chunk.  Returns the segment's size in bytes.
__device__ __forceinline__ uint32_t place_subs(const uint32_t* s_side, uint32_t m, uint32_t lane,
                                               bool any_stored, uint32_t* start, bool* in_block,
                                               uint32_t* tail_start, bool* tail_in_block) {
    uint32_t pos = 0;
    bool open = false;
    if (!any_stored) {
        // one Huffman block: positions are prefix sums of the token bits
        uint32_t total;
        const uint32_t ex = wave_excl_scan(s_side[lane], lane, &total);
        *start = lane == 0 ? 0u : 3u + ex;
        *in_block = lane != 0;
        pos = 3u + total;
        open = true;
    } else {
        *start = 0;
        *in_block = false;
        for (uint32_t s = 0; s < CODEC_NSUB; ++s) {
            const uint32_t n_s = min(CODEC_SUB, m - min(m, s * CODEC_SUB));
            if (s == lane) { *start = pos; *in_block = open; }
            if (n_s == 0u) continue;
            const uint32_t v = s_side[s];
            if (v == CODEC_STORED) {
                pos += (open ? 7u : 0u) + 3u;
                pos = ((pos + 7u) & ~7u) + 32u + 8u * n_s;
                open = false;
            } else {
                pos += (open ? 0u : 3u) + v;
                open = true;
            }
        }
    }
    *tail_start = pos;
    *tail_in_block = open;
    pos += (open ? 7u : 0u) + 3u;
    return ((pos + 7u) >> 3) + 4u;
}

// One wave per chunk: stages the chunk in LDS, marks the run starts, counts the token bits
// of every sub-chunk, chooses coded or stored per sub-chunk and for the chunk, builds the
// segment in LDS and writes it to the chunk's slot of the workspace together with its size.
// Two instances: OUT_DW = CODEC_OUT_SMALL (12 KiB of LDS for the segment, three waves per CU)
// takes every chunk first and passes those with a longer segment on to a list, which the
// instance with room for any segment (two waves per CU) works through.
constexpr uint32_t CODEC_OUT_SMALL = 3072;
constexpr uint32_t CODEC_OUT_FULL = CODEC_CHUNK / 4 + 8;
template <uint32_t OUT_DW>
__global__ __launch_bounds__(64) void deflate_chunk_kernel(
    const uint8_t* __restrict__ in, uint64_t n_bytes, uint32_t n_chunks,
    uint8_t* __restrict__ slots, uint32_t* __restrict__ seg_size, uint16_t* __restrict__ side,
    const uint32_t* __restrict__ list, uint32_t* __restrict__ long_list,
    uint32_t* __restrict__ long_count) {
    __shared__ __align__(16) uint32_t s_in[CODEC_CHUNK / 4];
    __shared__ uint32_t s_out[OUT_DW];
    __shared__ uint32_t s_mask[CODEC_NSUB * CODEC_MASKW];
    __shared__ uint32_t s_side[CODEC_NSUB];
    const uint32_t c = list ? list[blockIdx.x] : blockIdx.x, lane = threadIdx.x;
    const uint64_t base = (uint64_t)c * CODEC_CHUNK;
    const uint32_t m = (uint32_t)min((uint64_t)CODEC_CHUNK, n_bytes - min(n_bytes, base));
    const uint32_t last = c + 1u == n_chunks ? 1u : 0u;
    // stage: whole dwords coalesced, the ragged tail byte by byte, the rest zero
    uint32_t any_bits = m == CODEC_CHUNK ? 0u : 1u;    // stays 0 only for a full chunk of zeros
    if (m == CODEC_CHUNK) {
        // 32 loads of 16 bytes per lane, all in flight together
        const uint4* in128 = reinterpret_cast<const uint4*>(in + base);
        uint4 v[32];
#pragma unroll
        for (uint32_t u = 0; u < 32u; ++u) v[u] = in128[u * 64u + lane];
#pragma unroll
        for (uint32_t u = 0; u < 32u; ++u) {
            any_bits |= v[u].x | v[u].y | v[u].z | v[u].w;
            const uint32_t g = (u * 64u + lane) * 4u;
            const uint32_t l = g / CODEC_SUBW, j = g % CODEC_SUBW;
            *reinterpret_cast<uint4*>(&s_in[sub_word(l, j)]) = v[u];
        }
    } else {
        const uint32_t* in32 = reinterpret_cast<const uint32_t*>(in + base);
        for (uint32_t g = lane; g < CODEC_CHUNK / 4; g += 64u) {
            uint32_t v = 0;
            if (g * 4u + 4u <= m) {
                v = in32[g];
            } else {
                for (uint32_t k = 0; k < 4u; ++k)
                    if (g * 4u + k < m) v |= (uint32_t)in[base + g * 4u + k] << (8u * k);
            }
            s_in[sub_word(g / CODEC_SUBW, g % CODEC_SUBW)] = v;
        }
    }
    __syncthreads();
    const uint32_t n_l = min(CODEC_SUB, m - min(m, lane * CODEC_SUB));
    // Bit masks over the bytes of this lane's sub-chunk, 16 words each: S, byte i starts a run
    // (it differs from byte i - 1; position n_l counts as a start); G, byte i >= 144 (its
    // literal code has 9 bits).  From S: the bytes sent as literals (L: starts, and the
    // second and third byte of runs shorter than 4); a literal not followed by a literal
    // starts a run of 4 or more.
    uint32_t* mk = s_mask + lane * CODEC_MASKW;
    uint32_t tok_bits = 0;
    if (__ballot(any_bits != 0u) == 0ull) {
        // a chunk of zeros (common in sparse models): every sub-chunk is one literal and the
        // matches 258 + 253
#pragma unroll
        for (uint32_t a = 0; a < CODEC_MASKW; ++a) mk[a] = (a == 0 || a == CODEC_SUB / 32) ? 1u : 0u;
        tok_bits = 8u;
    } else {
        constexpr uint32_t NW = CODEC_SUB / 32;
        uint32_t S[NW + 1], G[NW];
        uint32_t carry = 0x100u;                       // no byte equals it: byte 0 starts a run
#pragma unroll
        for (uint32_t a = 0; a < NW; ++a) {
            uint32_t sw = 0, gw = 0;
            uint4 q4[2];
            q4[0] = *reinterpret_cast<const uint4*>(&s_in[sub_word(lane, a * 8u)]);
            q4[1] = *reinterpret_cast<const uint4*>(&s_in[sub_word(lane, a * 8u + 4u)]);
            const uint32_t ws[8] = {q4[0].x, q4[0].y, q4[0].z, q4[0].w, q4[1].x, q4[1].y, q4[1].z, q4[1].w};
#pragma unroll
            for (uint32_t b = 0; b < 8u; ++b) {
                const uint32_t w = ws[b];
                const uint32_t x = w ^ ((w << 8) | (carry & 0xffu));
                // bit 7 of every byte: the byte of x is not 0; the byte of w is >= 0x90
                uint32_t ne = ((((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u) >> 7;
                uint32_t ge = (w & (((w & 0x70707070u) + 0x70707070u)) & 0x80808080u) >> 7;
                ne = (ne | (ne >> 7) | (ne >> 14) | (ne >> 21)) & 0xfu;
                ge = (ge | (ge >> 7) | (ge >> 14) | (ge >> 21)) & 0xfu;
                if (a == 0 && b == 0) ne |= 1u;
                carry = w >> 24;
                sw |= ne << (4u * b);
                gw |= ge << (4u * b);
            }
            S[a] = sw;
            G[a] = gw;
        }
        S[NW] = 1u;                                    // position 512 ends the last run
        if (n_l < CODEC_SUB) {
#pragma unroll
            for (uint32_t a = 0; a < NW; ++a)
                if ((n_l >> 5) == a) S[a] |= 1u << (n_l & 31u);
        }
        uint32_t n_lit = 0, n_nine = 0;
#pragma unroll
        for (uint32_t a = 0; a < NW; ++a) {
            const uint32_t s0 = S[a], sp = a ? S[a - 1] : 0u, sn = S[a + 1];
            const uint32_t z0 = ~s0, zp = a ? ~S[a - 1] : 0u, zn = ~S[a + 1];
            const uint32_t s_b1 = (s0 << 1) | (sp >> 31), s_b2 = (s0 << 2) | (sp >> 30);   // bit p: S at p - 1, p - 2
            const uint32_t z_b1 = (z0 << 1) | (zp >> 31);
            const uint32_t s_f1 = (s0 >> 1) | (sn << 31), s_f2 = (s0 >> 2) | (sn << 30);   // bit p: S at p + 1, p + 2
            const uint32_t z_f1 = (z0 >> 1) | (zn << 31);
            const uint32_t valid = n_l >= 32u * (a + 1u) ? ~0u : (n_l <= 32u * a ? 0u : (1u << (n_l - 32u * a)) - 1u);
            const uint32_t lit = (s0 | (z0 & s_b1 & s_f1) | (z0 & s_b1 & z_f1 & s_f2) |
                                  (z0 & z_b1 & s_b2 & s_f1)) & valid;
            n_lit += (uint32_t)__popc(lit);
            n_nine += (uint32_t)__popc(lit & G[a]);
            const uint32_t end_bit = (n_l < CODEC_SUB && (n_l >> 5) == a) ? 1u << (n_l & 31u) : 0u;
            mk[a] = lit | end_bit;
        }
        mk[NW] = 1u;
        tok_bits = 8u * n_lit + n_nine;
    }
    // the matches of the runs of 4 or more: a literal whose next byte is not a literal starts
    // one (every byte of a shorter run is a literal); every lane reads only its own row
    {
        BitCounter cnt;
        for (uint32_t a = 0; a < CODEC_SUB / 32; ++a) {
            uint32_t mw = mk[a] & ~((mk[a] >> 1) | (mk[a + 1u] << 31));
            while (mw) {
                const uint32_t p = a * 32u + (uint32_t)__ffs((int)mw) - 1u;
                mw &= mw - 1u;
                if (p < n_l) put_matches(next_bit(mk, p) - p - 1u, cnt);
            }
        }
        tok_bits += cnt.bits;
    }
    const bool stored_sub = n_l > 0u && tok_bits > 8u * n_l + CODEC_MARGIN;
    const uint32_t my_side = stored_sub ? CODEC_STORED : tok_bits;
    s_side[lane] = my_side;
    __syncthreads();
    const bool any_stored = __ballot(stored_sub) != 0ull;
    uint32_t start, tail_start;
    bool in_block, tail_in_block;
    const uint32_t seg_bytes = place_subs(s_side, m, lane, any_stored, &start, &in_block,
                                          &tail_start, &tail_in_block);
    uint32_t* slot32 = reinterpret_cast<uint32_t*>(slots + (uint64_t)c * CODEC_SLOT);
    if (m + 5u <= seg_bytes) {
        // one stored block: header byte, LEN, NLEN, then the chunk, shifted by five bytes
        side[(uint64_t)c * CODEC_NSUB + lane] = 0;
        if (lane == 0) seg_size[c] = m + 5u;
        const uint32_t n_w = (m + 5u + 3u) / 4u;
        auto src = [&](uint32_t g) {               // dword g of the chunk (0 beyond it)
            return g < CODEC_CHUNK / 4 ? s_in[sub_word(g / CODEC_SUBW, g % CODEC_SUBW)] : 0u;
        };
        for (uint32_t k = lane; k < n_w; k += 64u) {
            uint32_t v;
            if (k == 0) v = last | (m << 8) | ((m ^ 0xffffu) << 24);
            else if (k == 1) v = ((m ^ 0xffffu) >> 8) | (src(0) << 8);
            else v = (src(k - 2) >> 24) | (src(k - 1) << 8);
            slot32[k] = v;
        }
        return;
    }
    if (OUT_DW < CODEC_OUT_FULL && (seg_bytes + 3u) / 4u > OUT_DW) {
        if (lane == 0) long_list[atomicAdd(long_count, 1u)] = c;   // for the other instance
        return;
    }
    side[(uint64_t)c * CODEC_NSUB + lane] = (uint16_t)my_side;
    if (lane == 0) seg_size[c] = seg_bytes;
    // bit range of this lane: to the next lane's start; lane 63 also writes the tail
    uint32_t end = __shfl_down(start, 1, 64);
    if (lane == 63u) end = seg_bytes * 8u;
    const uint32_t n_w = (seg_bytes + 3u) / 4u;
    for (uint32_t k = lane; k < n_w; k += 64u) s_out[k] = 0;
    __syncthreads();
    if (end > start) {
        BitWriter w(s_out, start);
        if (n_l > 0u && !stored_sub) {
            if (!in_block) w.put(2u, 3u);          // BFINAL = 0, BTYPE = 01
            encode_sub(s_in, mk, lane, n_l, w);
        } else if (n_l > 0u) {
            if (in_block) w.put(0u, 7u);           // end of the open block
            w.put(0u, 3u);                         // BFINAL = 0, BTYPE = 00
            const uint32_t at = start + (in_block ? 10u : 3u);
            w.put(0u, (8u - (at & 7u)) & 7u);
            w.put(n_l, 16u);
            w.put(n_l ^ 0xffffu, 16u);
            for (uint32_t j = 0; j < n_l / 4u; ++j) w.put(s_in[sub_word(lane, j)], 32u);
            for (uint32_t i = n_l & ~3u; i < n_l; ++i)
                w.put((s_in[sub_word(lane, i >> 2)] >> ((i & 3u) * 8u)) & 0xffu, 8u);
        }
        if (lane == 63u) {
            if (tail_in_block) w.put(0u, 7u);      // end of block
            w.put(last, 3u);                       // empty stored block: BFINAL, BTYPE = 00
            const uint32_t at = tail_start + (tail_in_block ? 10u : 3u);
            w.put(0u, (8u - (at & 7u)) & 7u);
            w.put(0x0000u, 16u);
            w.put(0xffffu, 16u);
        }
        w.finish();
    }
    __syncthreads();
    for (uint32_t k = lane; k < n_w; k += 64u) slot32[k] = s_out[k];
}

// Byte offsets of the segments: exclusive prefix sums of their sizes (one block).
__global__ __launch_bounds__(1024) void codec_scan_kernel(const uint32_t* __restrict__ seg_size,
                                                          uint32_t n_chunks,
                                                          uint64_t* __restrict__ seg_off,
                                                          uint64_t stream_cap,
                                                          uint64_t* __restrict__ result) {
    __shared__ uint64_t s_wave[16];
    __shared__ uint64_t s_carry;
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (uint32_t b0 = 0; b0 < n_chunks; b0 += 1024u) {
        const uint32_t i = b0 + threadIdx.x;
        const uint64_t v = i < n_chunks ? seg_size[i] : 0u;
        unsigned long long x = v;
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const unsigned long long y = __shfl_up(x, d, 64);
            if (lane >= d) x += y;
        }
        if (lane == 63u) s_wave[wid] = x;
        __syncthreads();
        uint64_t off = s_carry;
        for (uint32_t k = 0; k < wid; ++k) off += s_wave[k];
        if (i < n_chunks) seg_off[i] = off + x - v;
        __syncthreads();
        if (threadIdx.x == 1023u) s_carry = off + x;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        seg_off[n_chunks] = s_carry;
        result[0] = s_carry;
        result[1] = s_carry > stream_cap ? CODEC_CAPACITY : 0u;
    }
}

// Moves every segment from its slot to its place in the stream (one wave per chunk).  The
// slot is dword aligned, the destination is not: whole destination dwords are assembled
// from two source dwords, the ragged ends go byte by byte.
__global__ __launch_bounds__(64) void codec_pack_kernel(const uint8_t* __restrict__ slots,
                                                        const uint32_t* __restrict__ seg_size,
                                                        const uint64_t* __restrict__ seg_off,
                                                        const uint64_t* __restrict__ result,
                                                        uint8_t* __restrict__ stream) {
    if (result[1] != 0) return;                       // the stream does not fit: write nothing
    const uint32_t c = blockIdx.x, lane = threadIdx.x;
    const uint8_t* src = slots + (uint64_t)c * CODEC_SLOT;
    const uint32_t* src32 = reinterpret_cast<const uint32_t*>(src);
    uint8_t* dst = stream + seg_off[c];
    const uint32_t len = seg_size[c];
    const uint32_t head = min(len, (uint32_t)((4u - (reinterpret_cast<uintptr_t>(dst) & 3u)) & 3u));
    if (lane < head) dst[lane] = src[lane];
    const uint32_t n_w = (len - head) / 4u;
    uint32_t* dst32 = reinterpret_cast<uint32_t*>(dst + head);
    const uint32_t sh = head * 8u;
    for (uint32_t k = lane; k < n_w; k += 64u) {
        // bytes head + 4k .. head + 4k + 3 of the slot (its last dword + 1 is still inside it)
        const uint32_t lo = src32[k];
        dst32[k] = sh ? (lo >> sh) | (src32[k + 1] << (32u - sh)) : lo;
    }
    const uint32_t done = head + n_w * 4u;
    if (lane < len - done) dst[done + lane] = src[done + lane];
}

// Dwords of a segment kept in LDS by the three instances of the decoder: 7.5 KiB, 16 KiB
// and a whole segment.  The less LDS, the more chunks a CU works on at a time.
constexpr uint32_t CODEC_SEG_SMALL = 1920;
constexpr uint32_t CODEC_SEG_MEDIUM = 4096;
constexpr uint32_t CODEC_SEG_LARGE = (CODEC_SLOT + 3) / 4 + 3;
constexpr uint32_t CODEC_STAGE = 128;                  // output bytes per lane and stage
constexpr uint32_t CODEC_STAGE_W = CODEC_STAGE / 4;

// n <= 32 bits at bit position pos of the staged segment
__device__ __forceinline__ uint32_t seg_peek(const uint32_t* s_seg, uint32_t pos, uint32_t n) {
    const uint32_t w = pos >> 5, sh = pos & 31u;
    const uint64_t two = (uint64_t)s_seg[w] | ((uint64_t)s_seg[w + 1u] << 32);
    return (uint32_t)(two >> sh) & (n >= 32u ? ~0u : (1u << n) - 1u);
}
__device__ __forceinline__ uint32_t seg_byte(const uint32_t* s_seg, uint32_t b) {
    return (s_seg[b >> 2] >> ((b & 3u) * 8u)) & 0xffu;
}

// Dword j (0..31) of lane l's 128-byte piece of the stage image: the index of the 16-byte
// vector is XOR-ed with the lane, so that lanes at the same offset spread over the banks
// and a vector stays whole for the write-out.
__device__ __forceinline__ uint32_t img_word(uint32_t l, uint32_t j) {
    return l * CODEC_STAGE_W + ((((j >> 2) ^ l) & 7u) << 2) + (j & 3u);
}
__device__ __forceinline__ uint32_t img_byte(uint32_t l, uint32_t k) {   // byte k (0..127) of lane l's piece
    return img_word(l, k >> 2) * 4u + (k & 3u);
}

// What the next 9 bits of a fixed-Huffman block mean (RFC 1951 section 3.2.6), indexed by
// those bits as they come out of the stream (first bit = bit 0):
//   bits 0-4 bits used (a match: code + extra + 5 distance bits); bit 5 match; bit 6 not a
//   token (end of block, 286, 287); bits 8-16 the literal, or the match's base length;
//   bits 20-23 length of the code; bits 24-26 number of extra bits.
struct TokenTable {
    uint32_t v[512];
};
constexpr TokenTable make_token_table() {
    TokenTable t{};
    for (uint32_t r = 0; r < 512u; ++r) {
        uint32_t c9 = 0;                               // the 9 bits in code order
        for (uint32_t k = 0; k < 9u; ++k) c9 |= ((r >> k) & 1u) << (8u - k);
        uint32_t e = 0;
        if (c9 >= 0x190u) {                            // 9 bits: literals 144..255
            e = 9u | ((c9 - 0x100u) << 8);
        } else if ((c9 >> 1) >= 0x30u && (c9 >> 1) <= 0xBFu) {   // 8 bits: literals 0..143
            e = 8u | (((c9 >> 1) - 0x30u) << 8);
        } else {
            const bool seven = (c9 >> 2) <= 23u;       // 7 bits: 256..279; 8 bits: 280..287
            const uint32_t sym = seven ? 256u + (c9 >> 2) : 280u + (c9 >> 1) - 0xC0u;
            const uint32_t ncode = seven ? 7u : 8u;
            if (sym == 256u || sym > 285u) {
                e = ncode | 32u | 64u | (ncode << 20);
            } else {
                const uint32_t idx = sym - 257u;
                const uint32_t ex = (idx < 8u || idx == 28u) ? 0u : (idx - 4u) >> 2;
                const uint32_t lbase = idx < 8u ? 3u + idx : (idx == 28u ? 258u : 3u + ((4u + (idx & 3u)) << ex));
                e = (ncode + ex + 5u) | 32u | (lbase << 8) | (ncode << 20) | (ex << 24);
            }
        }
        t.v[r] = e;
    }
    return t;
}
static __device__ const TokenTable kTokenTable = make_token_table();

// One wave per chunk.  A chunk stored as one block is copied.  Otherwise the segment is
// staged in LDS and every lane finds its sub-chunk's place from the side information; the
// chunk is then produced in four stages of 128 bytes per sub-chunk: every lane decodes
// tokens (or copies stored bytes) into a zeroed LDS image of the stage, which is written
// out as whole 128-byte lines.  Three instances share the chunks by segment size (SEG_DW
// dwords of LDS for the segment); the smallest also takes the chunks stored as one block.
// The segment's size must be what the side information implies; anything but this
// library's own token set marks the stream as bad; no access leaves the stream or the
// output.
template <uint32_t SEG_DW, uint32_t SEG_MIN>
__global__ __launch_bounds__(64) void inflate_chunk_kernel(
    const uint8_t* __restrict__ stream, uint64_t stream_bytes, const uint64_t* __restrict__ seg_off,
    const uint16_t* __restrict__ side, uint64_t n_bytes, uint32_t n_chunks,
    uint8_t* __restrict__ out, uint64_t* __restrict__ result, const uint32_t* __restrict__ list) {
    __shared__ __align__(16) uint32_t s_img[CODEC_NSUB * CODEC_STAGE_W];
    __shared__ uint32_t s_seg[SEG_DW];
    __shared__ uint32_t s_tab[512];
    __shared__ uint32_t s_side[CODEC_NSUB];
    constexpr bool FIRST = SEG_MIN == 0;
    const uint32_t c = list ? list[blockIdx.x] : blockIdx.x, lane = threadIdx.x;   // list: the chunks of this instance
    const uint64_t base = (uint64_t)c * CODEC_CHUNK;
    const uint32_t m = (uint32_t)min((uint64_t)CODEC_CHUNK, n_bytes - min(n_bytes, base));
    const uint64_t s0 = seg_off[c], s1 = seg_off[c + 1];
    const uint32_t my_side = side[(uint64_t)c * CODEC_NSUB + lane];
    unsigned long long* status = reinterpret_cast<unsigned long long*>(&result[1]);
    if (s1 < s0 || s1 > stream_bytes || s1 - s0 < 5u || s1 - s0 > CODEC_SLOT) {
        if (FIRST && lane == 0) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
        return;
    }
    const uint32_t seg_len = (uint32_t)(s1 - s0);
    // The segment is read as dwords aligned to the stream's start.  The stream's last dword
    // may be partly beyond stream_bytes: an aligned dword never crosses a page, and what
    // lies beyond the segment is never interpreted.
    const uint32_t byte0 = (uint32_t)(s0 & 3u);
    const uint32_t* seg32 = reinterpret_cast<const uint32_t*>(stream + (s0 & ~(uint64_t)3u));
    const uint32_t max_w = (uint32_t)(((stream_bytes + 3u) / 4u) - (s0 >> 2)) - 1u;   // last readable dword
    const uint32_t seg_w = (byte0 + seg_len + 3u) / 4u + 2u;       // two more for the look-ahead
    const bool whole = __ballot(my_side != 0u) == 0ull;
    // the lists of the other instances are made from the first sub-chunk's side information
    if (whole != (__shfl(my_side, 0, 64) == 0u)) {
        if (FIRST && lane == 0) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
        return;
    }
    const uint32_t size_class = whole ? 0u : seg_w;
    if (size_class < SEG_MIN || size_class > SEG_DW) return;       // another instance's chunk
    uint8_t* dst = out + base;
    const uint32_t n_l = min(CODEC_SUB, m - min(m, lane * CODEC_SUB));
    if (whole) {
        // the whole chunk in one stored block
        uint32_t* dst32 = reinterpret_cast<uint32_t*>(dst);
        const uint8_t* seg = stream + s0;
        const uint32_t len = seg[1] | ((uint32_t)seg[2] << 8), nlen = seg[3] | ((uint32_t)seg[4] << 8);
        if (((seg[0] >> 1) & 3u) != 0u || len != m || (len ^ nlen) != 0xffffu || seg_len != m + 5u) {
            if (lane == 0) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
            return;
        }
        // output dword k = segment bytes 5 + 4k .. 5 + 4k + 3, assembled from two dwords
        const uint32_t sh = ((byte0 + 5u) & 3u) * 8u, w0 = (byte0 + 5u) >> 2;
        for (uint32_t k0 = 0; k0 < m / 4u; k0 += 64u * 8u) {
            uint32_t lo[8], hi[8];
#pragma unroll
            for (uint32_t u = 0; u < 8u; ++u) {
                const uint32_t w = w0 + k0 + u * 64u + lane;
                lo[u] = w <= max_w ? seg32[w] : 0u;
                hi[u] = w + 1u <= max_w ? seg32[w + 1u] : 0u;
            }
#pragma unroll
            for (uint32_t u = 0; u < 8u; ++u) {
                const uint32_t k = k0 + u * 64u + lane;
                if (k < m / 4u) dst32[k] = sh ? (lo[u] >> sh) | (hi[u] << (32u - sh)) : lo[u];
            }
        }
        if (lane < (m & 3u)) dst[(m & ~3u) + lane] = seg[5u + (m & ~3u) + lane];
        return;
    }
    const bool stored_sub = my_side == CODEC_STORED;
    bool ok = stored_sub ? n_l > 0u : (n_l > 0u ? my_side <= 8u * n_l + CODEC_MARGIN : my_side == 0u);
    s_side[lane] = ok ? my_side : 0u;
    for (uint32_t k = lane; k < seg_w; k += 64u) s_seg[k] = k <= max_w ? seg32[k] : 0u;
#pragma unroll
    for (uint32_t k = 0; k < 8u; ++k) s_tab[k * 64u + lane] = kTokenTable.v[k * 64u + lane];
    __syncthreads();
    const bool all_ok = __ballot(!ok) == 0ull;
    const bool any_stored = __ballot(stored_sub) != 0ull;
    uint32_t start, tail_start;
    bool in_block, tail_in_block;
    const uint32_t seg_bytes = place_subs(s_side, m, lane, any_stored, &start, &in_block,
                                          &tail_start, &tail_in_block);
    if (!all_ok || seg_bytes != seg_len) {
        if (lane == 0) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
        return;
    }
    const uint32_t bit0 = byte0 * 8u;
    // the structure around the sub-chunks: block headers, ends of blocks, the closing
    // empty stored block
    if (n_l > 0u) {
        if (!stored_sub && !in_block && seg_peek(s_seg, bit0 + start, 3u) != 2u) ok = false;
        if (stored_sub && seg_peek(s_seg, bit0 + start, in_block ? 10u : 3u) != 0u) ok = false;
    }
    if (lane == 63u) {
        const uint32_t last = c + 1u == n_chunks ? 1u : 0u;
        uint32_t at = bit0 + tail_start;
        if (tail_in_block) {
            if (seg_peek(s_seg, at, 7u) != 0u) ok = false;
            at += 7u;
        }
        if (seg_peek(s_seg, at, 3u) != last) ok = false;
        at = (at + 3u + 7u) & ~7u;
        if (seg_peek(s_seg, at, 32u) != 0xffff0000u) ok = false;
    }
    // per-lane decoder state, carried from stage to stage
    uint32_t i = 0;                                // bytes produced in this sub-chunk
    uint32_t pos = 0, end = 0, d0 = 0;             // token bits [pos, end), or first stored byte
    uint32_t prev = 0, pending = 0;                // pending: bytes of a run not yet produced
    if (stored_sub && ok) {
        // end-of-block of the open block (7 zero bits), header 000, padding, LEN, NLEN, bytes
        const uint32_t at = bit0 + start + (in_block ? 10u : 3u);
        const uint32_t b0 = ((at + 7u) >> 3);      // byte position of LEN, relative to seg32
        const uint32_t len = seg_byte(s_seg, b0) | (seg_byte(s_seg, b0 + 1u) << 8);
        const uint32_t nlen = seg_byte(s_seg, b0 + 2u) | (seg_byte(s_seg, b0 + 3u) << 8);
        if (len != n_l || (len ^ nlen) != 0xffffu) ok = false;
        d0 = b0 + 4u;
    } else if (ok) {
        pos = bit0 + start + (in_block ? 0u : 3u);
        end = pos + my_side;
    }
    uint8_t* img8 = reinterpret_cast<uint8_t*>(s_img);
    for (uint32_t st = 0; st < CODEC_SUB / CODEC_STAGE; ++st) {
        const uint32_t lo_b = st * CODEC_STAGE;
        const uint32_t hi_b = min(n_l, lo_b + CODEC_STAGE);     // this lane produces [i, hi_b)
#pragma unroll
        for (uint32_t j = 0; j < CODEC_STAGE_W / 4; ++j)
            reinterpret_cast<uint4*>(s_img)[j * CODEC_NSUB + lane] = make_uint4(0, 0, 0, 0);
        __syncthreads();
        if (stored_sub) {
            if (ok && hi_b > lo_b) {
                const uint32_t sh = (d0 & 3u) * 8u, w0 = (d0 + lo_b) >> 2;
                const uint32_t nw = (hi_b - lo_b) / 4u;
#pragma unroll 8
                for (uint32_t k = 0; k < nw; ++k) {
                    const uint32_t lo = s_seg[w0 + k];
                    s_img[img_word(lane, k)] = sh ? (lo >> sh) | (s_seg[w0 + k + 1u] << (32u - sh)) : lo;
                }
                for (uint32_t k = lo_b + nw * 4u; k < hi_b; ++k) img8[img_byte(lane, k - lo_b)] = (uint8_t)seg_byte(s_seg, d0 + k);
                i = hi_b;
            }
        } else {
            // what is left of a run that crossed the stage boundary
            if (ok && pending && i < hi_b) {
                const uint32_t k = min(pending, hi_b - i);
                if (prev)
                    for (uint32_t t = 0; t < k; ++t) img8[img_byte(lane, i - lo_b + t)] = (uint8_t)prev;
                i += k;
                pending -= k;
            }
            // one token per turn: the next 9 bits index the token table
            while (ok && i < hi_b) {
                if (pos >= end) { ok = false; break; }
                const uint32_t w = pos >> 5, sh = pos & 31u;
                const uint32_t x = (uint32_t)(((uint64_t)s_seg[w] | ((uint64_t)s_seg[w + 1u] << 32)) >> sh);
                const uint32_t t = s_tab[x & 511u];
                const uint32_t val = (t >> 8) & 0x1ffu;
                pos += t & 31u;
                if (!(t & 32u)) {
                    img8[img_byte(lane, i - lo_b)] = (uint8_t)val;
                    prev = val;
                    i += 1u;
                } else {
                    const uint32_t ncode = (t >> 20) & 15u, e = (t >> 24) & 7u;
                    const uint32_t len = val + ((x >> ncode) & ((1u << e) - 1u));
                    // a token, after a first byte, at distance 1, inside the sub-chunk
                    if ((t & 64u) || i == 0u || ((x >> (ncode + e)) & 31u) != 0u || len > n_l - i) {
                        ok = false;
                        break;
                    }
                    const uint32_t k = min(len, hi_b - i);
                    if (prev)                      // zero runs are already there
                        for (uint32_t u = 0; u < k; ++u) img8[img_byte(lane, i - lo_b + u)] = (uint8_t)prev;
                    i += k;
                    pending = len - k;
                }
            }
        }
        __syncthreads();
        // write-out: eight lanes per 128-byte line, eight lines per step
        if (m == CODEC_CHUNK) {
#pragma unroll
            for (uint32_t r = 0; r < CODEC_NSUB / 8u; ++r) {
                const uint32_t p = r * 8u + (lane >> 3), q = lane & 7u;     // piece, 16-byte vector
                const uint4 v = reinterpret_cast<const uint4*>(s_img)[p * 8u + ((q ^ p) & 7u)];
                *reinterpret_cast<uint4*>(dst + p * CODEC_SUB + lo_b + q * 16u) = v;
            }
        } else {
            for (uint32_t r = 0; r < CODEC_NSUB / 8u; ++r) {
                const uint32_t p = r * 8u + (lane >> 3), q = lane & 7u;
                const uint32_t n_p = min(CODEC_SUB, m - min(m, p * CODEC_SUB));
                const uint32_t valid = n_p - min(n_p, lo_b);            // bytes of this stage's piece
                if (q * 16u >= valid) continue;
                const uint4 v4 = reinterpret_cast<const uint4*>(s_img)[p * 8u + ((q ^ p) & 7u)];
                const uint32_t v[4] = {v4.x, v4.y, v4.z, v4.w};
                uint8_t* o = dst + p * CODEC_SUB + lo_b + q * 16u;
                if (q * 16u + 16u <= valid) {
                    *reinterpret_cast<uint4*>(o) = v4;
                } else {
                    for (uint32_t k = 0; q * 16u + k < valid; ++k) o[k] = (uint8_t)(v[k >> 2] >> (8u * (k & 3u)));
                }
            }
        }
        __syncthreads();
    }
    if (!ok || i != n_l || pending != 0u || (!stored_sub && pos != end))
        atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
}

__global__ void codec_clear_kernel(uint64_t* result) {
    result[0] = 0;
    result[1] = 0;
    result[2] = 0;      // lengths of the two chunk lists of the decoder
    result[3] = 0;
}

// Room for chunk lists, kept by the context and grown when a longer input comes.
static hipError_t codec_ensure_list(shifter_ctx* ctx, uint64_t entries) {
    if (ctx->codec_list_cap >= entries) return hipSuccess;
    if (ctx->d_codec_list) {
        hipError_t e = hipFree(ctx->d_codec_list);
        ctx->d_codec_list = nullptr;
        ctx->codec_list_cap = 0;
        if (e != hipSuccess) return e;
    }
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&ctx->d_codec_list), sizeof(uint32_t) * entries);
    if (e == hipSuccess) ctx->codec_list_cap = entries;
    return e;
}

// Waits (on an event) for the first instance and the length of its list.  Returns a HIP
// error code (0: fine).
int launch_deflate(shifter_ctx* ctx, const uint8_t* d_in, uint64_t n_bytes, uint32_t n_chunks,
                   uint8_t* d_work, uint8_t* d_stream, uint64_t stream_cap, uint64_t* d_seg_off,
                   uint16_t* d_sub_bits) {
    hipError_t e = codec_ensure_list(ctx, 2ull * n_chunks);
    if (e != hipSuccess) return (int)e;
    uint32_t* seg_size = reinterpret_cast<uint32_t*>(d_work);
    uint8_t* slots = d_work + codec_slots_offset(n_chunks);
    uint32_t* long_count = reinterpret_cast<uint32_t*>(ctx->d_codec + 2);
    codec_clear_kernel<<<1, 1, 0, ctx->stream>>>(ctx->d_codec);
    {
        ProfileScope ps(ctx, K_DEFLATE_CHUNK);
        deflate_chunk_kernel<CODEC_OUT_SMALL><<<n_chunks, 64, 0, ctx->stream>>>(
            d_in, n_bytes, n_chunks, slots, seg_size, d_sub_bits, nullptr, ctx->d_codec_list, long_count);
        if ((e = hipMemcpyAsync(ctx->h_codec + 2, ctx->d_codec + 2, sizeof(uint64_t), hipMemcpyDeviceToHost,
                                ctx->stream)) != hipSuccess) return (int)e;
        if ((e = hipEventRecord(ctx->codec_ev, ctx->stream)) != hipSuccess) return (int)e;
        if ((e = hipEventSynchronize(ctx->codec_ev)) != hipSuccess) return (int)e;
        const uint32_t n_long = (uint32_t)ctx->h_codec[2];
        if (n_long)
            deflate_chunk_kernel<CODEC_OUT_FULL><<<n_long, 64, 0, ctx->stream>>>(
                d_in, n_bytes, n_chunks, slots, seg_size, d_sub_bits, ctx->d_codec_list, nullptr, nullptr);
    }
    {
        ProfileScope ps(ctx, K_CODEC_SCAN);
        codec_scan_kernel<<<1, 1024, 0, ctx->stream>>>(seg_size, n_chunks, d_seg_off, stream_cap,
                                                       ctx->d_codec);
    }
    ProfileScope ps(ctx, K_CODEC_PACK);
    codec_pack_kernel<<<n_chunks, 64, 0, ctx->stream>>>(slots, seg_size, d_seg_off, ctx->d_codec,
                                                        d_stream);
    return 0;
}

// Lists of the chunks whose segments need the medium and the large instance of the decoder
// (the same rule as inside the instances); counts in result[2] and result[3].
__global__ __launch_bounds__(BLOCK) void codec_classify_kernel(
    uint64_t stream_bytes, const uint64_t* __restrict__ seg_off, const uint16_t* __restrict__ side,
    uint32_t n_chunks, uint32_t* __restrict__ list_medium, uint32_t* __restrict__ list_large,
    uint64_t* __restrict__ result) {
    const uint32_t c = blockIdx.x * BLOCK + threadIdx.x;
    if (c >= n_chunks) return;
    const uint64_t s0 = seg_off[c], s1 = seg_off[c + 1];
    if (s1 < s0 || s1 > stream_bytes || s1 - s0 < 5u || s1 - s0 > CODEC_SLOT) return;   // the first instance reports it
    if (side[(uint64_t)c * CODEC_NSUB] == 0u) return;                                     // one stored block
    const uint32_t seg_w = ((uint32_t)(s0 & 3u) + (uint32_t)(s1 - s0) + 3u) / 4u + 2u;
    if (seg_w > CODEC_SEG_MEDIUM)
        list_large[atomicAdd(reinterpret_cast<uint32_t*>(&result[3]), 1u)] = c;
    else if (seg_w > CODEC_SEG_SMALL)
        list_medium[atomicAdd(reinterpret_cast<uint32_t*>(&result[2]), 1u)] = c;
}

// Streams of this many chunks or more get lists for the two larger instances (a block that
// finds a chunk is not its own costs about 2 us of a CU slot); for shorter ones all three
// instances visit every chunk and the call needs no wait in the middle.
constexpr uint32_t CODEC_LIST_MIN_CHUNKS = 16384;

// Returns a HIP error code (0: fine).
int launch_inflate(shifter_ctx* ctx, const uint8_t* d_stream, uint64_t stream_bytes,
                   const uint64_t* d_seg_off, const uint16_t* d_sub_bits, uint64_t n_bytes,
                   uint32_t n_chunks, uint8_t* d_out) {
    const bool lists = n_chunks >= CODEC_LIST_MIN_CHUNKS;
    uint32_t *list_medium = nullptr, *list_large = nullptr;
    if (lists) {
        hipError_t e0 = codec_ensure_list(ctx, 2ull * n_chunks);
        if (e0 != hipSuccess) return (int)e0;
        list_medium = ctx->d_codec_list;
        list_large = ctx->d_codec_list + n_chunks;
    }
    codec_clear_kernel<<<1, 1, 0, ctx->stream>>>(ctx->d_codec);
    ProfileScope ps(ctx, K_INFLATE_CHUNK);
    uint32_t n_medium = n_chunks, n_large = n_chunks;
    if (lists) {
        codec_classify_kernel<<<(n_chunks + BLOCK - 1) / BLOCK, BLOCK, 0, ctx->stream>>>(
            stream_bytes, d_seg_off, d_sub_bits, n_chunks, list_medium, list_large, ctx->d_codec);
        hipError_t e = hipMemcpyAsync(ctx->h_codec + 2, ctx->d_codec + 2, 2 * sizeof(uint64_t),
                                      hipMemcpyDeviceToHost, ctx->stream);
        if (e != hipSuccess) return (int)e;
        if ((e = hipEventRecord(ctx->codec_ev, ctx->stream)) != hipSuccess) return (int)e;
    }
    // The three instances are independent: the first runs on the caller's stream, the other
    // two on streams of the context that fork from it and join it again (all of default
    // priority), so that their blocks share the CUs instead of queueing behind each other.
    hipError_t e = hipEventRecord(ctx->codec_fork, ctx->stream);
    if (e != hipSuccess) return (int)e;
    // the first instance (it skips the chunks of the other two) runs while the counts travel
    inflate_chunk_kernel<CODEC_SEG_SMALL, 0><<<n_chunks, 64, 0, ctx->stream>>>(
        d_stream, stream_bytes, d_seg_off, d_sub_bits, n_bytes, n_chunks, d_out, ctx->d_codec, nullptr);
    if (lists) {
        if ((e = hipEventSynchronize(ctx->codec_ev)) != hipSuccess) return (int)e;
        n_medium = (uint32_t)ctx->h_codec[2];
        n_large = (uint32_t)ctx->h_codec[3];
    }
    if (n_large) {
        if ((e = hipStreamWaitEvent(ctx->codec_aux[0], ctx->codec_fork, 0)) != hipSuccess) return (int)e;
        inflate_chunk_kernel<CODEC_SEG_LARGE, CODEC_SEG_MEDIUM + 1><<<n_large, 64, 0, ctx->codec_aux[0]>>>(
            d_stream, stream_bytes, d_seg_off, d_sub_bits, n_bytes, n_chunks, d_out, ctx->d_codec, list_large);
        if ((e = hipEventRecord(ctx->codec_join[0], ctx->codec_aux[0])) != hipSuccess) return (int)e;
        if ((e = hipStreamWaitEvent(ctx->stream, ctx->codec_join[0], 0)) != hipSuccess) return (int)e;
    }
    if (n_medium) {
        if ((e = hipStreamWaitEvent(ctx->codec_aux[1], ctx->codec_fork, 0)) != hipSuccess) return (int)e;
        inflate_chunk_kernel<CODEC_SEG_MEDIUM, CODEC_SEG_SMALL + 1><<<n_medium, 64, 0, ctx->codec_aux[1]>>>(
            d_stream, stream_bytes, d_seg_off, d_sub_bits, n_bytes, n_chunks, d_out, ctx->d_codec, list_medium);
        if ((e = hipEventRecord(ctx->codec_join[1], ctx->codec_aux[1])) != hipSuccess) return (int)e;
        if ((e = hipStreamWaitEvent(ctx->stream, ctx->codec_join[1], 0)) != hipSuccess) return (int)e;
    }
    return 0;
}

}  // namespace shifter
