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
//   - a mark per coded sub-chunk, so that four lanes share it: for each of its later three
//     quarters of 128 bytes, the token bits of the quarter before (11 bits) and how far past
//     the quarter's start its first literal lies (9 bits); a run's matches go with the
//     literal that starts the run, so a lane never needs another lane's bytes.
// Any inflater reads the stream; the encoder and the decoder here work with one block of
// 256 threads per chunk, four lanes per sub-chunk.
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

constexpr uint32_t CODEC_Q = 4;                               // lanes per sub-chunk
constexpr uint32_t CODEC_QB = CODEC_SUB / CODEC_Q;            // 128 bytes of a sub-chunk per lane
constexpr uint32_t CODEC_QW = CODEC_QB / 32;                  // 4 mask words per lane
constexpr uint32_t CODEC_THREADS = CODEC_NSUB * CODEC_Q;      // 256: one block per chunk
constexpr uint32_t CODEC_LOOP_GRID = 1536;                    // blocks of an instance that walks a list

// Run-start bits (bit i: byte 32 a + i of sub-chunk l differs from the byte before it;
// byte 0 always starts a run) and the bits of the bytes >= 144 (their literal code has 9
// bits) of mask word a.
__device__ __forceinline__ void mask_word(const uint32_t* s_in, uint32_t l, uint32_t a, uint32_t* s_out,
                                          uint32_t* g_out) {
    uint32_t carry = a ? s_in[sub_word(l, a * 8u - 1u)] >> 24 : 0u;
    uint32_t sw = 0, gw = 0;
    uint4 q4[2];
    q4[0] = *reinterpret_cast<const uint4*>(&s_in[sub_word(l, a * 8u)]);
    q4[1] = *reinterpret_cast<const uint4*>(&s_in[sub_word(l, a * 8u + 4u)]);
    const uint32_t ws[8] = {q4[0].x, q4[0].y, q4[0].z, q4[0].w, q4[1].x, q4[1].y, q4[1].z, q4[1].w};
#pragma unroll
    for (uint32_t b = 0; b < 8u; ++b) {
        const uint32_t w = ws[b];
        const uint32_t x = w ^ ((w << 8) | carry);
        // bit 7 of every byte: the byte of x is not 0; the byte of w is >= 0x90
        uint32_t ne = ((((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u) >> 7;
        uint32_t ge = (w & (((w & 0x70707070u) + 0x70707070u)) & 0x80808080u) >> 7;
        ne = (ne | (ne >> 7) | (ne >> 14) | (ne >> 21)) & 0xfu;
        ge = (ge | (ge >> 7) | (ge >> 14) | (ge >> 21)) & 0xfu;
        carry = w >> 24;
        sw |= ne << (4u * b);
        gw |= ge << (4u * b);
    }
    if (a == 0) sw |= 1u;
    *s_out = sw;
    *g_out = gw;
}

// Tokens of sub-chunk l whose literal lies in [p, p_end): every literal there, and the
// matches of the run it starts (which may reach past p_end).  mk: one bit per byte sent as
// a literal, and a set bit at the sub-chunk's length.  p must be a literal's position.
template <class Sink>
__device__ __forceinline__ void encode_range(const uint32_t* s_in, const uint32_t* mk, uint32_t l,
                                             uint32_t p, uint32_t p_end, Sink& sink) {
    while (p < p_end) {
        const uint32_t q = next_bit(mk, p);
        const uint32_t b = (s_in[sub_word(l, p >> 2)] >> ((p & 3u) * 8u)) & 0xffu;
        uint32_t code;
        const uint32_t nb = literal_code(b, &code);
        sink.put(code, nb);
        if (q - p >= 4u) put_matches(q - p - 1u, sink);
        p = q;
    }
}

// One block of 256 threads per chunk, four lanes per sub-chunk (one per 128 bytes): stages
// the chunk in LDS, marks the bytes sent as literals, counts the token bits of every
// quarter (a run's matches count with the literal that starts it), chooses coded or stored
// per sub-chunk and for the chunk, builds the segment in LDS - every lane appends the tokens
// of its quarter at the bit position the counts give it - and writes it to the chunk's slot
// of the workspace together with its size.  The same counts are the decoder's marks.
// Two instances: OUT_DW = CODEC_OUT_SMALL (12 KiB of LDS for the segment) takes every chunk
// first and passes those with a longer segment on to a list, which the instance with room
// for any segment walks (LISTED: a fixed grid, block b takes entries b, b + grid, ...).
constexpr uint32_t CODEC_OUT_SMALL = 3072;
constexpr uint32_t CODEC_OUT_FULL = CODEC_CHUNK / 4 + 8;

struct DeflateShared {
    uint32_t* in;       // CODEC_CHUNK / 4
    uint32_t* out;      // OUT_DW
    uint32_t* mask;     // CODEC_NSUB * CODEC_MASKW
    uint32_t* side;     // CODEC_NSUB
    uint32_t* start;    // CODEC_NSUB: bit 31 = a block is open there
    uint32_t* misc;     // segment bytes, tail start, tail in block
};

template <uint32_t OUT_DW>
__device__ __forceinline__ void deflate_chunk(
    const DeflateShared& sh, uint32_t c, const uint8_t* __restrict__ in, uint64_t n_bytes, uint32_t n_chunks,
    uint8_t* __restrict__ slots, uint32_t* __restrict__ seg_size, uint16_t* __restrict__ side,
    uint64_t* __restrict__ marks, uint32_t* __restrict__ long_list, uint32_t* __restrict__ long_count) {
    uint32_t* s_in = sh.in;
    const uint32_t tid = threadIdx.x, l = tid >> 2, q = tid & 3u;
    const uint64_t base = (uint64_t)c * CODEC_CHUNK;
    const uint32_t m = (uint32_t)min((uint64_t)CODEC_CHUNK, n_bytes - min(n_bytes, base));
    const uint32_t last = c + 1u == n_chunks ? 1u : 0u;
    // stage: whole dwords coalesced, the ragged tail byte by byte, the rest zero
    uint32_t any_bits = m == CODEC_CHUNK ? 0u : 1u;    // stays 0 only for a full chunk of zeros
    if (m == CODEC_CHUNK) {
        // 8 loads of 16 bytes per thread, all in flight together
        const uint4* in128 = reinterpret_cast<const uint4*>(in + base);
        uint4 v[8];
#pragma unroll
        for (uint32_t u = 0; u < 8u; ++u) v[u] = in128[u * CODEC_THREADS + tid];
#pragma unroll
        for (uint32_t u = 0; u < 8u; ++u) {
            any_bits |= v[u].x | v[u].y | v[u].z | v[u].w;
            const uint32_t g = (u * CODEC_THREADS + tid) * 4u;
            *reinterpret_cast<uint4*>(&s_in[sub_word(g / CODEC_SUBW, g % CODEC_SUBW)]) = v[u];
        }
    } else {
        const uint32_t* in32 = reinterpret_cast<const uint32_t*>(in + base);
        for (uint32_t g = tid; g < CODEC_CHUNK / 4; g += CODEC_THREADS) {
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
    const bool zero_chunk = __syncthreads_or(any_bits != 0u) == 0;
    const uint32_t n_l = min(CODEC_SUB, m - min(m, l * CODEC_SUB));      // bytes of this sub-chunk
    const uint32_t p_lo = min(q * CODEC_QB, n_l), p_hi = min(p_lo + CODEC_QB, n_l);   // this lane's quarter
    // Bit masks over the bytes of this lane's quarter, 4 words: S, byte i starts a run (it
    // differs from byte i - 1; position n_l counts as a start); G, byte i >= 144.  From S:
    // the bytes sent as literals (starts, and the second and third byte of runs shorter
    // than 4); a literal not followed by a literal starts a run of 4 or more.
    uint32_t* mk = sh.mask + l * CODEC_MASKW;
    const uint32_t a0 = q * CODEC_QW;
    uint32_t tok_bits = 0;
    if (zero_chunk) {
        // a chunk of zeros (common in sparse models): every sub-chunk is one literal and the
        // matches 258 + 253
#pragma unroll
        for (uint32_t j = 0; j < CODEC_QW; ++j) mk[a0 + j] = (a0 + j == 0u) ? 1u : 0u;
        if (q == CODEC_Q - 1u) mk[CODEC_SUB / 32] = 1u;
        tok_bits = q == 0u ? 8u : 0u;
    } else {
        constexpr uint32_t NW = CODEC_SUB / 32;
        // S[1 .. 4], G[1 .. 4]: this lane's words; S[0] and S[5]: the words next to them, from
        // the neighbouring lanes of the sub-chunk (the lanes of a sub-chunk are neighbours in
        // the wavefront); position 512 ends the last run
        uint32_t S[CODEC_QW + 2], G[CODEC_QW + 2];
#pragma unroll
        for (uint32_t k = 1; k <= CODEC_QW; ++k) {
            const uint32_t a = a0 + k - 1u;
            mask_word(s_in, l, a, &S[k], &G[k]);
            if (n_l < CODEC_SUB && (n_l >> 5) == a) S[k] |= 1u << (n_l & 31u);
        }
        {
            const uint32_t from_left = __shfl_up(S[CODEC_QW], 1, CODEC_Q);
            const uint32_t from_right = __shfl_down(S[1], 1, CODEC_Q);
            S[0] = q == 0u ? 0u : from_left;
            S[CODEC_QW + 1] = q == CODEC_Q - 1u ? 1u : from_right;
            G[0] = G[CODEC_QW + 1] = 0;
        }
        uint32_t n_lit = 0, n_nine = 0;
#pragma unroll
        for (uint32_t j = 0; j < CODEC_QW; ++j) {
            const uint32_t a = a0 + j;
            const uint32_t s0 = S[j + 1], sp = a ? S[j] : 0u, sn = S[j + 2];
            const uint32_t z0 = ~s0, zp = a ? ~S[j] : 0u, zn = ~S[j + 2];
            const uint32_t s_b1 = (s0 << 1) | (sp >> 31), s_b2 = (s0 << 2) | (sp >> 30);   // bit p: S at p - 1, p - 2
            const uint32_t z_b1 = (z0 << 1) | (zp >> 31);
            const uint32_t s_f1 = (s0 >> 1) | (sn << 31), s_f2 = (s0 >> 2) | (sn << 30);   // bit p: S at p + 1, p + 2
            const uint32_t z_f1 = (z0 >> 1) | (zn << 31);
            const uint32_t valid = n_l >= 32u * (a + 1u) ? ~0u : (n_l <= 32u * a ? 0u : (1u << (n_l - 32u * a)) - 1u);
            const uint32_t lit = (s0 | (z0 & s_b1 & s_f1) | (z0 & s_b1 & z_f1 & s_f2) |
                                  (z0 & z_b1 & s_b2 & s_f1)) & valid;
            n_lit += (uint32_t)__popc(lit);
            n_nine += (uint32_t)__popc(lit & G[j + 1]);
            const uint32_t end_bit = (n_l < CODEC_SUB && (n_l >> 5) == a) ? 1u << (n_l & 31u) : 0u;
            mk[a] = lit | end_bit;
        }
        if (q == CODEC_Q - 1u) mk[NW] = 1u;
        tok_bits = 8u * n_lit + n_nine;
    }
    __syncthreads();
    // the matches of the runs of 4 or more that start in this quarter: a literal whose next
    // byte is not a literal starts one (every byte of a shorter run is a literal)
    {
        BitCounter cnt;
        for (uint32_t j = 0; j < CODEC_QW; ++j) {
            const uint32_t a = a0 + j;
            uint32_t mw = mk[a] & ~((mk[a] >> 1) | (mk[a + 1u] << 31));
            while (mw) {
                const uint32_t p = a * 32u + (uint32_t)__ffs((int)mw) - 1u;
                mw &= mw - 1u;
                if (p < n_l) put_matches(next_bit(mk, p) - p - 1u, cnt);
            }
        }
        tok_bits += cnt.bits;
    }
    // bits before this quarter's tokens (the lanes of a sub-chunk are neighbours), and the
    // sub-chunk's total
    uint32_t before = 0, total = tok_bits;
    {
        const uint32_t t1 = __shfl_up(tok_bits, 1, CODEC_Q), t2 = __shfl_up(tok_bits, 2, CODEC_Q),
                       t3 = __shfl_up(tok_bits, 3, CODEC_Q);
        if (q >= 1u) before += t1;
        if (q >= 2u) before += t2;
        if (q >= 3u) before += t3;
        total = __shfl(before + tok_bits, CODEC_Q - 1u, CODEC_Q);
    }
    // first literal at or after the quarter's start (the sub-chunk's length if there is none)
    uint32_t first = p_lo;
    if (q > 0u && p_lo < n_l && !((mk[p_lo >> 5] >> (p_lo & 31u)) & 1u)) first = next_bit(mk, p_lo);
    const bool stored_sub = n_l > 0u && total > 8u * n_l + CODEC_MARGIN;
    const uint32_t my_side = stored_sub ? CODEC_STORED : total;
    // the decoder's mark: per later quarter the bits of the quarter before it and how far
    // past its start its first literal lies
    uint64_t mark = 0;
    {
        const uint32_t prev_bits = __shfl_up(tok_bits, 1, CODEC_Q);
        const uint64_t field = q ? (uint64_t)(prev_bits | ((first - p_lo) << 11)) << (20u * (q - 1u)) : 0ull;
        const uint64_t f1 = __shfl_down(field, 1, CODEC_Q), f2 = __shfl_down(field, 2, CODEC_Q),
                       f3 = __shfl_down(field, 3, CODEC_Q);
        mark = (n_l > 0u && !stored_sub) ? (f1 | f2 | f3) : 0ull;          // meaningful in lane q = 0
    }
    if (q == 0u) sh.side[l] = my_side;
    const bool any_stored = __syncthreads_or(stored_sub) != 0;
    if (tid < CODEC_NSUB) {
        uint32_t start, tail_start;
        bool in_block, tail_in_block;
        const uint32_t sb = place_subs(sh.side, m, tid, any_stored, &start, &in_block, &tail_start,
                                       &tail_in_block);
        sh.start[tid] = start | (in_block ? 0x80000000u : 0u);
        if (tid == 0) {
            sh.misc[0] = sb;
            sh.misc[1] = tail_start;
            sh.misc[2] = tail_in_block ? 1u : 0u;
        }
    }
    __syncthreads();
    const uint32_t seg_bytes = sh.misc[0];
    uint32_t* slot32 = reinterpret_cast<uint32_t*>(slots + (uint64_t)c * CODEC_SLOT);
    if (m + 5u <= seg_bytes) {
        // one stored block: header byte, LEN, NLEN, then the chunk, shifted by five bytes
        if (q == 0u) {
            side[(uint64_t)c * CODEC_NSUB + l] = 0;
            marks[(uint64_t)c * CODEC_NSUB + l] = 0;
        }
        if (tid == 0) seg_size[c] = m + 5u;
        const uint32_t n_w = (m + 5u + 3u) / 4u;
        auto src = [&](uint32_t g) {               // dword g of the chunk (0 beyond it)
            return g < CODEC_CHUNK / 4 ? s_in[sub_word(g / CODEC_SUBW, g % CODEC_SUBW)] : 0u;
        };
        for (uint32_t k = tid; k < n_w; k += CODEC_THREADS) {
            uint32_t v;
            if (k == 0) v = last | (m << 8) | ((m ^ 0xffffu) << 24);
            else if (k == 1) v = ((m ^ 0xffffu) >> 8) | (src(0) << 8);
            else v = (src(k - 2) >> 24) | (src(k - 1) << 8);
            slot32[k] = v;
        }
        return;
    }
    if (OUT_DW < CODEC_OUT_FULL && (seg_bytes + 3u) / 4u > OUT_DW) {
        if (tid == 0) long_list[atomicAdd(long_count, 1u)] = c;   // for the other instance
        return;
    }
    if (q == 0u) {
        side[(uint64_t)c * CODEC_NSUB + l] = (uint16_t)my_side;
        marks[(uint64_t)c * CODEC_NSUB + l] = mark;
    }
    if (tid == 0) seg_size[c] = seg_bytes;
    const uint32_t n_w = (seg_bytes + 3u) / 4u;
    for (uint32_t k = tid; k < n_w; k += CODEC_THREADS) sh.out[k] = 0;
    __syncthreads();
    const uint32_t start = sh.start[l] & 0x7fffffffu;
    const bool in_block = (sh.start[l] >> 31) != 0u;
    if (n_l > 0u && !stored_sub) {
        // lane 0 opens the block if none is open; every lane appends its quarter's tokens
        const uint32_t tok0 = start + (in_block ? 0u : 3u);
        BitWriter w(sh.out, q == 0u ? start : tok0 + before);
        if (q == 0u && !in_block) w.put(2u, 3u);          // BFINAL = 0, BTYPE = 01
        encode_range(s_in, mk, l, first, p_hi, w);
        w.finish();
    } else if (n_l > 0u) {
        // stored: lane 0 closes the open block and writes the header, every lane its bytes
        const uint32_t at = start + (in_block ? 10u : 3u);
        const uint32_t data_bit = ((at + 7u) & ~7u) + 32u;
        if (q == 0u) {
            BitWriter w(sh.out, start);
            if (in_block) w.put(0u, 7u);                  // end of the open block
            w.put(0u, 3u);                                // BFINAL = 0, BTYPE = 00
            w.put(0u, (8u - (at & 7u)) & 7u);
            w.put(n_l, 16u);
            w.put(n_l ^ 0xffffu, 16u);
            w.finish();
        }
        if (p_hi > p_lo) {
            BitWriter w(sh.out, data_bit + 8u * p_lo);
            const uint32_t nq = p_hi - p_lo;
            for (uint32_t j = 0; j < nq / 4u; ++j) w.put(s_in[sub_word(l, p_lo / 4u + j)], 32u);
            for (uint32_t i = p_lo + (nq & ~3u); i < p_hi; ++i)
                w.put((s_in[sub_word(l, i >> 2)] >> ((i & 3u) * 8u)) & 0xffu, 8u);
            w.finish();
        }
    }
    if (tid == CODEC_THREADS - 1u) {
        const uint32_t tail_start = sh.misc[1];
        const bool tail_in_block = sh.misc[2] != 0u;
        BitWriter w(sh.out, tail_start);
        if (tail_in_block) w.put(0u, 7u);                 // end of block
        w.put(last, 3u);                                  // empty stored block: BFINAL, BTYPE = 00
        const uint32_t at = tail_start + (tail_in_block ? 10u : 3u);
        w.put(0u, (8u - (at & 7u)) & 7u);
        w.put(0x0000u, 16u);
        w.put(0xffffu, 16u);
        w.finish();
    }
    __syncthreads();
    for (uint32_t k = tid; k < n_w; k += CODEC_THREADS) slot32[k] = sh.out[k];
}

template <uint32_t OUT_DW, bool LISTED>
__global__ __launch_bounds__(CODEC_THREADS) void deflate_chunk_kernel(
    const uint8_t* __restrict__ in, uint64_t n_bytes, uint32_t n_chunks,
    uint8_t* __restrict__ slots, uint32_t* __restrict__ seg_size, uint16_t* __restrict__ side,
    uint64_t* __restrict__ marks, const uint32_t* __restrict__ list, uint32_t* __restrict__ long_list,
    uint32_t* __restrict__ long_count) {
    __shared__ __align__(16) uint32_t s_in[CODEC_CHUNK / 4];
    __shared__ uint32_t s_out[OUT_DW];
    __shared__ uint32_t s_mask[CODEC_NSUB * CODEC_MASKW];
    __shared__ uint32_t s_side[CODEC_NSUB];
    __shared__ uint32_t s_start[CODEC_NSUB];
    __shared__ uint32_t s_misc[4];
    const DeflateShared sh{s_in, s_out, s_mask, s_side, s_start, s_misc};
    if (!LISTED) {
        deflate_chunk<OUT_DW>(sh, blockIdx.x, in, n_bytes, n_chunks, slots, seg_size, side, marks, long_list,
                              long_count);
    } else {
        const uint32_t n_list = *long_count;               // written by the instance before this one
        for (uint32_t it = blockIdx.x; it < n_list; it += gridDim.x) {
            deflate_chunk<OUT_DW>(sh, list[it], in, n_bytes, n_chunks, slots, seg_size, side, marks, nullptr,
                                  nullptr);
            __syncthreads();
        }
    }
}

// Byte offsets of the segments: exclusive prefix sums of their sizes (one block).  A row is
// 64 consecutive chunks, one per lane.  Every wavefront first sums its rows (every 16th),
// eight rows' loads in flight together and nothing shared but the row sums in LDS; then one
// block-wide scan over the thread totals of the row sums (a thread owns a run of rows); then
// the wavefronts visit their rows again and write the offsets: the row's base from the
// owner's total and the rows before it in the run, plus a scan across the lanes.  Three
// barriers per SCAN_ROWS_MAX rows (2 GiB of input), whatever the number of chunks below.
constexpr uint32_t SCAN_ROWS_MAX = 1024;
__global__ __launch_bounds__(1024) void codec_scan_kernel(const uint32_t* __restrict__ seg_size,
                                                          uint32_t n_chunks,
                                                          uint64_t* __restrict__ seg_off,
                                                          uint64_t stream_cap,
                                                          uint64_t* __restrict__ result) {
    __shared__ uint32_t s_row[SCAN_ROWS_MAX];           // a row's sizes sum to less than 2^32
    __shared__ uint64_t s_tbase[1024];                  // exclusive prefix of the threads' runs
    __shared__ uint64_t s_wave[16];
    const uint32_t lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    constexpr uint32_t R = 8;
    uint64_t carry = 0;                                 // the same in every thread
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += SCAN_ROWS_MAX * 64u) {
        const uint32_t n_here = min(n_chunks - c0, SCAN_ROWS_MAX * 64u);
        const uint32_t* size = seg_size + c0;
        const uint32_t rows = (n_here + 63u) / 64u;
        const uint32_t rpt = (rows + 1023u) / 1024u;    // rows per thread in the scan
        for (uint32_t j0 = wid; j0 < rows; j0 += 16u * R) {
            uint32_t v[R];
#pragma unroll
            for (uint32_t u = 0; u < R; ++u) {
                const uint32_t i = (j0 + 16u * u) * 64u + lane;       // rows j0, j0 + 16, ...
                v[u] = i < n_here ? size[i] : 0u;
            }
#pragma unroll
            for (uint32_t u = 0; u < R; ++u) {
                uint32_t x = v[u];
                for (uint32_t d = 32; d > 0; d >>= 1) x += __shfl_down(x, d, 64);
                if (lane == 0 && j0 + 16u * u < rows) s_row[j0 + 16u * u] = x;
            }
        }
        __syncthreads();
        {
            uint64_t mine = 0;
            for (uint32_t i = 0; i < rpt; ++i) {
                const uint32_t j = threadIdx.x * rpt + i;
                if (j < rows) mine += s_row[j];
            }
            unsigned long long x = mine;
            for (uint32_t d = 1; d < 64; d <<= 1) {
                const unsigned long long y = __shfl_up(x, d, 64);
                if (lane >= d) x += y;
            }
            if (lane == 63u) s_wave[wid] = x;
            __syncthreads();
            uint64_t off = carry, total = 0;
            for (uint32_t k = 0; k < 16u; ++k) {
                const uint64_t w = s_wave[k];
                if (k < wid) off += w;
                total += w;
            }
            s_tbase[threadIdx.x] = off + x - mine;
            carry += total;
        }
        __syncthreads();
        for (uint32_t j0 = wid; j0 < rows; j0 += 16u * R) {
            uint32_t v[R];
#pragma unroll
            for (uint32_t u = 0; u < R; ++u) {
                const uint32_t i = (j0 + 16u * u) * 64u + lane;
                v[u] = i < n_here ? size[i] : 0u;
            }
#pragma unroll
            for (uint32_t u = 0; u < R; ++u) {
                const uint32_t j = j0 + 16u * u, i = j * 64u + lane;
                if (j < rows) {                             // the same in every lane
                    const uint32_t owner = j / rpt;
                    uint64_t base = s_tbase[owner];
                    for (uint32_t r = owner * rpt; r < j; ++r) base += s_row[r];
                    uint32_t x = v[u];
                    for (uint32_t d = 1; d < 64; d <<= 1) {
                        const uint32_t y = __shfl_up(x, d, 64);
                        if (lane >= d) x += y;
                    }
                    if (i < n_here) seg_off[(uint64_t)c0 + i] = base + x - v[u];
                }
            }
        }
        __syncthreads();                                // s_row and s_tbase are free again
    }
    if (threadIdx.x == 0) {
        seg_off[n_chunks] = carry;
        result[0] = carry;
        result[1] = carry > stream_cap ? CODEC_CAPACITY : 0u;
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

// Dwords of a segment kept in LDS by the three instances of the decoder: 4.5 KiB (with the
// chunk's image and the token table just under 40 KiB, four blocks per CU), 16 KiB and a
// whole segment.  The less LDS, the more chunks a CU works on at a time.
constexpr uint32_t CODEC_SEG_SMALL = 1152;
constexpr uint32_t CODEC_SEG_MEDIUM = 4096;
constexpr uint32_t CODEC_SEG_LARGE = (CODEC_SLOT + 3) / 4 + 3;
// n <= 32 bits at bit position pos of the staged segment
__device__ __forceinline__ uint32_t seg_peek(const uint32_t* s_seg, uint32_t pos, uint32_t n) {
    const uint32_t w = pos >> 5, sh = pos & 31u;
    const uint64_t two = (uint64_t)s_seg[w] | ((uint64_t)s_seg[w + 1u] << 32);
    return (uint32_t)(two >> sh) & (n >= 32u ? ~0u : (1u << n) - 1u);
}
__device__ __forceinline__ uint32_t seg_byte(const uint32_t* s_seg, uint32_t b) {
    return (s_seg[b >> 2] >> ((b & 3u) * 8u)) & 0xffu;
}

// What the next 9 bits of a fixed-Huffman block mean (RFC 1951 section 3.2.6), indexed by
// those bits as they come out of the stream (first bit = bit 0):
//   bits 0-4 bits used (a match: code + extra + 5 distance bits); bit 5 match; bit 6 not a
//   token (end of block, 286, 287); bits 7-15 the base length (1 for a literal); bits 16-23
//   the literal; bits 24-27 length of a match's code; bits 28-30 its number of extra bits.
// With these a literal reads as a match of length 1 of itself, and one sequence of
// operations without a branch serves both.
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
            e = 9u | (1u << 7) | ((c9 - 0x100u) << 16);
        } else if ((c9 >> 1) >= 0x30u && (c9 >> 1) <= 0xBFu) {   // 8 bits: literals 0..143
            e = 8u | (1u << 7) | (((c9 >> 1) - 0x30u) << 16);
        } else {
            const bool seven = (c9 >> 2) <= 23u;       // 7 bits: 256..279; 8 bits: 280..287
            const uint32_t sym = seven ? 256u + (c9 >> 2) : 280u + (c9 >> 1) - 0xC0u;
            const uint32_t ncode = seven ? 7u : 8u;
            if (sym == 256u || sym > 285u) {
                e = ncode | 32u | 64u | (ncode << 24);
            } else {
                const uint32_t idx = sym - 257u;
                const uint32_t ex = (idx < 8u || idx == 28u) ? 0u : (idx - 4u) >> 2;
                const uint32_t lbase = idx < 8u ? 3u + idx : (idx == 28u ? 258u : 3u + ((4u + (idx & 3u)) << ex));
                e = (ncode + ex + 5u) | 32u | (lbase << 7) | (ncode << 24) | (ex << 28);
            }
        }
        t.v[r] = e;
    }
    return t;
}
static __device__ const TokenTable kTokenTable = make_token_table();

// Byte k of sub-chunk l in the LDS image of a chunk (rows rotated like the encoder's).
__device__ __forceinline__ uint32_t img_byte(uint32_t l, uint32_t k) {
    return sub_word(l, k >> 2) * 4u + (k & 3u);
}

struct InflateShared {
    uint32_t* img;      // CODEC_CHUNK / 4: the chunk being produced
    uint32_t* seg;      // SEG_DW: the segment
    uint32_t* tab;      // 512: token table
    uint32_t* side;     // CODEC_NSUB
    uint32_t* start;    // CODEC_NSUB: bit 31 = a block is open there
    uint32_t* misc;     // segment bytes, tail start, tail in block
};

// One block of 256 threads per chunk, four lanes per sub-chunk.  A chunk stored as one block
// is copied.  Otherwise the segment is staged in LDS, every sub-chunk's place follows from
// the side information and every lane's from the sub-chunk's mark: lane q decodes the tokens
// from bit b_q on (or copies its 128 stored bytes) into a zeroed LDS image of the chunk,
// which is then written out as whole lines.  Three instances share the chunks by segment
// size (SEG_DW dwords of LDS for the segment); the smallest visits every chunk and also
// takes those stored as one block, the other two walk lists.  The segment's size must be
// what the side information implies, every lane must end exactly where the next one
// starts, and anything but this library's own token set marks the stream as bad; no access
// leaves the stream, the staged segment, the image or the output.
template <uint32_t SEG_DW, uint32_t SEG_MIN>
__device__ __forceinline__ void inflate_chunk(
    const InflateShared& sh, uint32_t c, const uint8_t* __restrict__ stream, uint64_t stream_bytes,
    const uint64_t* __restrict__ seg_off, const uint16_t* __restrict__ side,
    const uint64_t* __restrict__ marks, uint64_t n_bytes, uint32_t n_chunks, uint8_t* __restrict__ out,
    uint64_t* __restrict__ result) {
    constexpr bool FIRST = SEG_MIN == 0;
    // The instance of the short segments (chunks that are mostly zeros) keeps no image of
    // the chunk: it writes the chunk's zeros to memory at once, 16 bytes per thread and
    // store, and after the block's barrier every lane stores its few non-zero bytes one by
    // one on top.  Without the 32 KiB image many more blocks fit a compute unit, and the
    // zeros are on their way while the segment is still being fetched.
    constexpr bool DIRECT = SEG_DW == CODEC_SEG_SMALL;
    const uint32_t tid = threadIdx.x, l = tid >> 2, q = tid & 3u;
    const uint64_t base = (uint64_t)c * CODEC_CHUNK;
    const uint32_t m = (uint32_t)min((uint64_t)CODEC_CHUNK, n_bytes - min(n_bytes, base));
    const uint64_t s0 = seg_off[c], s1 = seg_off[c + 1];
    unsigned long long* status = reinterpret_cast<unsigned long long*>(&result[1]);
    if (s1 < s0 || s1 > stream_bytes || s1 - s0 < 5u || s1 - s0 > CODEC_SLOT) {
        if (FIRST && tid == 0) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
        return;
    }
    const uint32_t my_side = side[(uint64_t)c * CODEC_NSUB + l];
    const uint32_t side0 = side[(uint64_t)c * CODEC_NSUB];
    const uint32_t seg_len = (uint32_t)(s1 - s0);
    // The segment is read as dwords aligned to the stream's start.  The stream's last dword
    // may be partly beyond stream_bytes: an aligned dword never crosses a page, and what
    // lies beyond the segment is never interpreted.
    const uint32_t byte0 = (uint32_t)(s0 & 3u);
    const uint32_t* seg32 = reinterpret_cast<const uint32_t*>(stream + (s0 & ~(uint64_t)3u));
    const uint32_t max_w = (uint32_t)(((stream_bytes + 3u) / 4u) - (s0 >> 2)) - 1u;   // last readable dword
    const uint32_t seg_w = (byte0 + seg_len + 3u) / 4u + 2u;       // two more for the look-ahead
    // One stored block iff the first sub-chunk's side information is 0 (the lists of the
    // other instances are made from it too); every thread then checks that its own
    // sub-chunk agrees: a coded or stored sub-chunk never has 0, a chunk stored whole has
    // nothing else.
    const bool whole = side0 == 0u;
    const uint32_t size_class = whole ? 0u : seg_w;
    if (size_class < SEG_MIN || size_class > SEG_DW) return;       // another instance's chunk
    uint8_t* dst = out + base;
    const uint32_t n_l = min(CODEC_SUB, m - min(m, l * CODEC_SUB));
    if (whole) {
        // the whole chunk in one stored block
        uint32_t* dst32 = reinterpret_cast<uint32_t*>(dst);
        const uint8_t* seg = stream + s0;
        const uint32_t len = seg[1] | ((uint32_t)seg[2] << 8), nlen = seg[3] | ((uint32_t)seg[4] << 8);
        if (my_side != 0u) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
        if (((seg[0] >> 1) & 3u) != 0u || len != m || (len ^ nlen) != 0xffffu || seg_len != m + 5u) {
            if (tid == 0) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
            return;
        }
        // output dword k = segment bytes 5 + 4k .. 5 + 4k + 3, assembled from two dwords
        const uint32_t shb = ((byte0 + 5u) & 3u) * 8u, w0 = (byte0 + 5u) >> 2;
        for (uint32_t k0 = 0; k0 < m / 4u; k0 += CODEC_THREADS * 8u) {
            uint32_t lo[8], hi[8];
#pragma unroll
            for (uint32_t u = 0; u < 8u; ++u) {
                const uint32_t w = w0 + k0 + u * CODEC_THREADS + tid;
                lo[u] = w <= max_w ? seg32[w] : 0u;
                hi[u] = w + 1u <= max_w ? seg32[w + 1u] : 0u;
            }
#pragma unroll
            for (uint32_t u = 0; u < 8u; ++u) {
                const uint32_t k = k0 + u * CODEC_THREADS + tid;
                if (k < m / 4u) dst32[k] = shb ? (lo[u] >> shb) | (hi[u] << (32u - shb)) : lo[u];
            }
        }
        if (tid < (m & 3u)) dst[(m & ~3u) + tid] = seg[5u + (m & ~3u) + tid];
        return;
    }
    const uint64_t mark = marks[(uint64_t)c * CODEC_NSUB + l];
    const bool stored_sub = my_side == CODEC_STORED;
    bool ok = stored_sub ? n_l > 0u : (n_l > 0u ? my_side <= 8u * n_l + CODEC_MARGIN : my_side == 0u);
    // The first wavefront, one lane per sub-chunk, works out where every sub-chunk's part of
    // the segment starts while the others stage the segment and clear the image: one barrier
    // before the decoding, one after it.
    if (tid < CODEC_NSUB) {
        const uint32_t n_s = min(CODEC_SUB, m - min(m, tid * CODEC_SUB));
        const uint32_t v = side[(uint64_t)c * CODEC_NSUB + tid];
        const bool st = v == CODEC_STORED;
        const bool ok_s = st ? n_s > 0u : (n_s > 0u ? v != 0u && v <= 8u * n_s + CODEC_MARGIN : v == 0u);
        sh.side[tid] = ok_s ? v : 0u;
        // the lanes exchange within their own wavefront only: order the LDS accesses
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const bool any_stored = __ballot(st) != 0ull;
        const bool all_ok = __ballot(!ok_s) == 0ull;
        uint32_t start, tail_start;
        bool in_block, tail_in_block;
        const uint32_t sb = place_subs(sh.side, m, tid, any_stored, &start, &in_block, &tail_start,
                                       &tail_in_block);
        sh.start[tid] = start | (in_block ? 0x80000000u : 0u);
        if (tid == 0) {
            sh.misc[0] = all_ok ? sb : 0xffffffffu;      // never a segment's size
            sh.misc[1] = tail_start;
            sh.misc[2] = tail_in_block ? 1u : 0u;
        }
    }
    for (uint32_t k = tid; k < seg_w; k += CODEC_THREADS) sh.seg[k] = k <= max_w ? seg32[k] : 0u;
    sh.tab[tid] = kTokenTable.v[tid];
    sh.tab[tid + CODEC_THREADS] = kTokenTable.v[tid + CODEC_THREADS];
    if (DIRECT) {
        if (m == CODEC_CHUNK) {
#pragma unroll
            for (uint32_t j = 0; j < CODEC_CHUNK / 16 / CODEC_THREADS; ++j)
                *reinterpret_cast<uint4*>(dst + (j * CODEC_THREADS + tid) * 16u) = make_uint4(0, 0, 0, 0);
        } else {
            for (uint32_t g = tid; g * 16u < m; g += CODEC_THREADS) {
                if (g * 16u + 16u <= m) *reinterpret_cast<uint4*>(dst + g * 16u) = make_uint4(0, 0, 0, 0);
                else for (uint32_t k = g * 16u; k < m; ++k) dst[k] = 0;
            }
        }
    } else {
#pragma unroll
        for (uint32_t j = 0; j < CODEC_CHUNK / 16 / CODEC_THREADS; ++j)
            reinterpret_cast<uint4*>(sh.img)[j * CODEC_THREADS + tid] = make_uint4(0, 0, 0, 0);
    }
    // orders the block's accesses to the image, and (DIRECT) its zeros in memory before the
    // bytes its lanes store on top of them
    __syncthreads();
    if (sh.misc[0] != seg_len) {
        if (tid == 0) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
        return;
    }
    const uint32_t* s_seg = sh.seg;
    const uint32_t bit0 = byte0 * 8u;
    const uint32_t start = sh.start[l] & 0x7fffffffu;
    const bool in_block = (sh.start[l] >> 31) != 0u;
    // the structure around the sub-chunks: block headers, ends of blocks, the closing
    // empty stored block
    if (n_l > 0u && q == 0u) {
        if (!stored_sub && !in_block && seg_peek(s_seg, bit0 + start, 3u) != 2u) ok = false;
        if (stored_sub && seg_peek(s_seg, bit0 + start, in_block ? 10u : 3u) != 0u) ok = false;
    }
    if (tid == CODEC_THREADS - 1u) {
        const uint32_t last = c + 1u == n_chunks ? 1u : 0u;
        uint32_t at = bit0 + sh.misc[1];
        if (sh.misc[2]) {
            if (seg_peek(s_seg, at, 7u) != 0u) ok = false;
            at += 7u;
        }
        if (seg_peek(s_seg, at, 3u) != last) ok = false;
        at = (at + 3u + 7u) & ~7u;
        if (seg_peek(s_seg, at, 32u) != 0xffff0000u) ok = false;
    }
    uint8_t* img8 = reinterpret_cast<uint8_t*>(sh.img);
    const uint32_t p_lo = min(q * CODEC_QB, n_l), p_hi = min(p_lo + CODEC_QB, n_l);
    if (stored_sub) {
        // end-of-block of the open block (7 zero bits), header 000, padding, LEN, NLEN, bytes
        const uint32_t at = bit0 + start + (in_block ? 10u : 3u);
        const uint32_t b0 = ((at + 7u) >> 3);      // byte position of LEN, relative to seg32
        const uint32_t len = seg_byte(s_seg, b0) | (seg_byte(s_seg, b0 + 1u) << 8);
        const uint32_t nlen = seg_byte(s_seg, b0 + 2u) | (seg_byte(s_seg, b0 + 3u) << 8);
        if (len != n_l || (len ^ nlen) != 0xffffu || mark != 0ull) ok = false;
        if (ok && p_hi > p_lo) {
            const uint32_t d0 = b0 + 4u + p_lo;    // this lane's first byte
            const uint32_t shb = (d0 & 3u) * 8u, w0 = d0 >> 2, nw = (p_hi - p_lo) / 4u;
            uint32_t* out32 = reinterpret_cast<uint32_t*>(dst + l * CODEC_SUB + p_lo);   // DIRECT: 128-byte aligned
#pragma unroll 8
            for (uint32_t k = 0; k < nw; ++k) {
                const uint32_t lo = s_seg[w0 + k];
                const uint32_t v = shb ? (lo >> shb) | (s_seg[w0 + k + 1u] << (32u - shb)) : lo;
                if (DIRECT) out32[k] = v;
                else sh.img[sub_word(l, p_lo / 4u + k)] = v;
            }
            for (uint32_t k = p_lo + nw * 4u; k < p_hi; ++k) {
                const uint8_t v = (uint8_t)seg_byte(s_seg, d0 + k - p_lo);
                if (DIRECT) dst[l * CODEC_SUB + k] = v;
                else img8[img_byte(l, k)] = v;
            }
        }
    } else if (n_l > 0u) {
        // this lane's range from the mark: bits [b_lo, b_hi) of the sub-chunk's tokens make
        // bytes [o_lo, o_hi)
        uint32_t b_lo = 0, b_hi = my_side, o_lo = 0, o_hi = n_l, b_acc = 0;
#pragma unroll
        for (uint32_t j = 1; j < CODEC_Q; ++j) {
            const uint32_t field = (uint32_t)(mark >> (20u * (j - 1u))) & 0xfffffu;
            b_acc += field & 0x7ffu;
            const uint32_t o_j = min(j * CODEC_QB, n_l) + (field >> 11);
            if (j == q) { b_lo = b_acc; o_lo = o_j; }
            if (j == q + 1u) { b_hi = b_acc; o_hi = o_j; }
        }
        if ((mark >> 60) != 0ull || b_lo > b_hi || b_hi > my_side || o_lo > o_hi || o_hi > n_l || o_lo < p_lo) ok = false;
        if (ok) {
            uint32_t pos = bit0 + start + (in_block ? 0u : 3u) + b_lo;
            const uint32_t end = pos + (b_hi - b_lo);
            uint32_t i = o_lo, prev = 0x100u;      // 0x100: no literal of this lane yet
            const uint32_t row = l * CODEC_SUB, rot = 16u * l;   // image byte of offset k: row + ((k + rot) & 511)
            // a 64-bit window of the token bits in two registers, sh bits of it used up
            uint32_t nextw = (pos >> 5) + 2u, sh_bits = pos & 31u;
            uint32_t w_lo = s_seg[pos >> 5], w_hi = s_seg[(pos >> 5) + 1u];
            uint32_t bad_bits = 0;
            // Up to two tokens per turn, without branches but for the stores: the table gives
            // a token's bits, kind and value, and a literal reads as a match of length 1 of
            // itself; when the token behind it is a literal (three quarters of all tokens are,
            // in half-empty data) that one is taken in the same turn (a third one gained 1 %).  Offsets are not checked
            // on the way: a store wraps inside its sub-chunk's row of the image, offsets only
            // grow, and the end must come out exactly right.
            while (pos < end) {
                const uint32_t x = __builtin_amdgcn_alignbit(w_hi, w_lo, sh_bits);
                const uint32_t t = sh.tab[x & 511u];
                const uint32_t nb = t & 31u;
                const uint32_t t2 = sh.tab[(x >> nb) & 511u];              // at most 18 of the 32 bits are used
                const uint32_t mm = 0u - ((t >> 5) & 1u);                  // all ones for a match
                const uint32_t len = ((t >> 7) & 0x1ffu) + __builtin_amdgcn_ubfe(x, (t >> 24) & 15u, t >> 28);
                const uint32_t byte = ((t >> 16) & 0xffu) | (prev & mm);    // a match repeats the byte before it
                // not a token of this library's set; a match before any literal of this lane, or
                // at a distance other than 1
                bad_bits |= (t & 64u) | ((__builtin_amdgcn_ubfe(x, nb - 5u, 5u) | (prev >> 8)) & mm);
                if ((byte & 0xffu) != 0u) {                                 // zeros are already there
                    if (DIRECT) {
                        // no image: straight to memory, inside the sub-chunk and the output
                        for (uint32_t u = 0; u < len; ++u) {
                            const uint32_t at = row + ((i + u) & (CODEC_SUB - 1u));
                            if (at < m) dst[at] = (uint8_t)byte;
                        }
                    } else {
                        img8[row + ((i + rot) & (CODEC_SUB - 1u))] = (uint8_t)byte;
                        for (uint32_t u = 1; u < len; ++u) img8[row + ((i + u + rot) & (CODEC_SUB - 1u))] = (uint8_t)byte;
                    }
                }
                i += len;
                // the second token: a literal that starts before the lane's last bit
                const bool two = (t2 & 0x60u) == 0u && pos + nb < end;
                const uint32_t byte2 = (t2 >> 16) & 0xffu;
                if (two && byte2 != 0u) {
                    if (DIRECT) {
                        const uint32_t at = row + (i & (CODEC_SUB - 1u));
                        if (at < m) dst[at] = (uint8_t)byte2;
                    } else {
                        img8[row + ((i + rot) & (CODEC_SUB - 1u))] = (uint8_t)byte2;
                    }
                }
                const uint32_t used = nb + (two ? t2 & 31u : 0u);          // at most 18 + 9 bits
                prev = two ? byte2 : byte;
                i += two ? 1u : 0u;
                pos += used;
                sh_bits += used;
                const uint32_t w_new = s_seg[min(nextw, SEG_DW - 1u)];
                const bool take = sh_bits >= 32u;
                w_lo = take ? w_hi : w_lo;
                w_hi = take ? w_new : w_hi;
                nextw += take ? 1u : 0u;
                sh_bits &= 31u;
            }
            if (bad_bits) ok = false;
            if (pos != end || i != o_hi) ok = false;
        }
    } else if (mark != 0ull) {
        ok = false;
    }
    const bool fine = __syncthreads_and(ok) != 0;
    if (!fine) {
        if (tid == 0) atomicOr(status, (unsigned long long)CODEC_BAD_STREAM);
        return;
    }
    if (DIRECT) return;
    // write-out: 16 bytes per thread and step, whole lines per wave
    if (m == CODEC_CHUNK) {
#pragma unroll
        for (uint32_t r = 0; r < CODEC_CHUNK / 16 / CODEC_THREADS; ++r) {
            const uint32_t g = r * CODEC_THREADS + tid;                 // 16-byte vector of the chunk
            const uint4 v = *reinterpret_cast<const uint4*>(&sh.img[sub_word(g >> 5, (g & 31u) * 4u)]);
            *reinterpret_cast<uint4*>(dst + g * 16u) = v;
        }
    } else {
        for (uint32_t r = 0; r < CODEC_CHUNK / 16 / CODEC_THREADS; ++r) {
            const uint32_t g = r * CODEC_THREADS + tid;
            if (g * 16u >= m) continue;
            const uint4 v4 = *reinterpret_cast<const uint4*>(&sh.img[sub_word(g >> 5, (g & 31u) * 4u)]);
            if (g * 16u + 16u <= m) {
                *reinterpret_cast<uint4*>(dst + g * 16u) = v4;
            } else {
                const uint32_t v[4] = {v4.x, v4.y, v4.z, v4.w};
                for (uint32_t k = 0; g * 16u + k < m; ++k) dst[g * 16u + k] = (uint8_t)(v[k >> 2] >> (8u * (k & 3u)));
            }
        }
    }
}

template <uint32_t SEG_DW, uint32_t SEG_MIN>
__global__ __launch_bounds__(CODEC_THREADS, SEG_DW == CODEC_SEG_SMALL ? 5 : (SEG_DW == CODEC_SEG_MEDIUM ? 3 : 2))
void inflate_chunk_kernel(
    const uint8_t* __restrict__ stream, uint64_t stream_bytes, const uint64_t* __restrict__ seg_off,
    const uint16_t* __restrict__ side, const uint64_t* __restrict__ marks, uint64_t n_bytes, uint32_t n_chunks,
    uint8_t* __restrict__ out, uint64_t* __restrict__ result, const uint32_t* __restrict__ list,
    const uint32_t* __restrict__ list_count) {
    __shared__ __align__(16) uint32_t s_img[SEG_DW == CODEC_SEG_SMALL ? 4 : CODEC_CHUNK / 4];   // none for the short segments
    __shared__ uint32_t s_seg[SEG_DW];
    __shared__ uint32_t s_tab[512];
    __shared__ uint32_t s_side[CODEC_NSUB];
    __shared__ uint32_t s_start[CODEC_NSUB];
    __shared__ uint32_t s_misc[4];
    const InflateShared sh{s_img, s_seg, s_tab, s_side, s_start, s_misc};
    if (!list) {
        inflate_chunk<SEG_DW, SEG_MIN>(sh, blockIdx.x, stream, stream_bytes, seg_off, side, marks, n_bytes,
                                       n_chunks, out, result);
    } else {
        const uint32_t n_list = *list_count;               // written by the classifying kernel
        for (uint32_t it = blockIdx.x; it < n_list; it += gridDim.x) {
            inflate_chunk<SEG_DW, SEG_MIN>(sh, list[it], stream, stream_bytes, seg_off, side, marks, n_bytes,
                                           n_chunks, out, result);
            __syncthreads();
        }
    }
}

__global__ void codec_clear_kernel(uint64_t* result) {
    result[0] = 0;
    result[1] = 0;
    result[2] = 0;      // lengths of the two chunk lists of the decoder, or of the encoder's one
    result[3] = 0;
}

// The call's outcome (stream bytes, status bits) into the pinned mirror the host reads after
// its wait; the result words are then cleared for the next call (zero after use: the next
// call needs no clearing launch of its own).
__global__ void codec_publish_kernel(uint64_t* __restrict__ result, uint64_t* __restrict__ mirror) {
    mirror[0] = result[0];
    mirror[1] = result[1];
    result[0] = 0;
    result[1] = 0;
    result[2] = 0;
    result[3] = 0;
}

// The result words are zero when a call starts: the context allocates them cleared and every
// call's last kernel leaves them so.  Only a call that could not enqueue all of its kernels
// leaves them in doubt; the call after it clears them itself.
static void codec_begin(shifter_ctx* ctx) {
    if (ctx->codec_dirty) codec_clear_kernel<<<1, 1, 0, ctx->stream>>>(ctx->d_codec);
    ctx->codec_dirty = true;
}
static void codec_end(shifter_ctx* ctx) {
    codec_publish_kernel<<<1, 1, 0, ctx->stream>>>(ctx->d_codec, ctx->dev_codec_mirror);
    if (hipPeekAtLastError() == hipSuccess) ctx->codec_dirty = false;
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

// Kernels only, nothing waited for.  Returns a HIP error code (0: fine).
int launch_deflate(shifter_ctx* ctx, const uint8_t* d_in, uint64_t n_bytes, uint32_t n_chunks,
                   uint8_t* d_work, uint8_t* d_stream, uint64_t stream_cap, uint64_t* d_seg_off,
                   uint16_t* d_sub_bits, uint64_t* d_sub_marks) {
    hipError_t e = codec_ensure_list(ctx, 2ull * n_chunks);
    if (e != hipSuccess) return (int)e;
    uint32_t* seg_size = reinterpret_cast<uint32_t*>(d_work);
    uint8_t* slots = d_work + codec_slots_offset(n_chunks);
    uint32_t* long_count = reinterpret_cast<uint32_t*>(ctx->d_codec + 2);
    codec_begin(ctx);
    {
        ProfileScope ps(ctx, K_DEFLATE_CHUNK);
        deflate_chunk_kernel<CODEC_OUT_SMALL, false><<<n_chunks, CODEC_THREADS, 0, ctx->stream>>>(
            d_in, n_bytes, n_chunks, slots, seg_size, d_sub_bits, d_sub_marks, nullptr, ctx->d_codec_list,
            long_count);
        // the chunks whose segment did not fit the first instance's LDS: a fixed grid walks
        // the list the first instance left, however long it is
        deflate_chunk_kernel<CODEC_OUT_FULL, true>
            <<<std::min(n_chunks, CODEC_LOOP_GRID), CODEC_THREADS, 0, ctx->stream>>>(
                d_in, n_bytes, n_chunks, slots, seg_size, d_sub_bits, d_sub_marks, ctx->d_codec_list, nullptr,
                long_count);
    }
    {
        ProfileScope ps(ctx, K_CODEC_SCAN);
        codec_scan_kernel<<<1, 1024, 0, ctx->stream>>>(seg_size, n_chunks, d_seg_off, stream_cap,
                                                       ctx->d_codec);
    }
    {
        ProfileScope ps(ctx, K_CODEC_PACK);
        codec_pack_kernel<<<n_chunks, 64, 0, ctx->stream>>>(slots, seg_size, d_seg_off, ctx->d_codec,
                                                            d_stream);
    }
    codec_end(ctx);
    return 0;
}

// Lists of the chunks whose segments need the medium and the large instance of the decoder
// (the same rule as inside the instances); counts in result[2] and result[3].  One atomic
// per block and list (atomics to one address take their turns, about 10 ns each): the
// wavefronts' counts meet in LDS and share the range the block reserves.
constexpr uint32_t CLASSIFY_THREADS = 1024;
__global__ __launch_bounds__(CLASSIFY_THREADS) void codec_classify_kernel(
    uint64_t stream_bytes, const uint64_t* __restrict__ seg_off, const uint16_t* __restrict__ side,
    uint32_t n_chunks, uint32_t* __restrict__ list_medium, uint32_t* __restrict__ list_large,
    uint64_t* __restrict__ result) {
    constexpr uint32_t WAVES = CLASSIFY_THREADS / 64u;
    __shared__ uint32_t s_cnt[2][WAVES], s_base[2];
    const uint32_t c = blockIdx.x * CLASSIFY_THREADS + threadIdx.x, lane = threadIdx.x & 63u, wid = threadIdx.x >> 6;
    uint32_t seg_w = 0;
    if (c < n_chunks) {
        const uint64_t s0 = seg_off[c], s1 = seg_off[c + 1];
        // a broken offset is reported by the first instance; one stored block is its chunk too
        if (!(s1 < s0 || s1 > stream_bytes || s1 - s0 < 5u || s1 - s0 > CODEC_SLOT) &&
            side[(uint64_t)c * CODEC_NSUB] != 0u)
            seg_w = ((uint32_t)(s0 & 3u) + (uint32_t)(s1 - s0) + 3u) / 4u + 2u;
    }
    const bool large = seg_w > CODEC_SEG_MEDIUM, medium = seg_w > CODEC_SEG_SMALL && !large;
    const uint64_t votes[2] = {__ballot(medium), __ballot(large)};
    if (lane == 0) {
        s_cnt[0][wid] = (uint32_t)__popcll(votes[0]);
        s_cnt[1][wid] = (uint32_t)__popcll(votes[1]);
    }
    __syncthreads();
    if (threadIdx.x < 2u) {
        uint32_t total = 0;
        for (uint32_t w = 0; w < WAVES; ++w) total += s_cnt[threadIdx.x][w];
        s_base[threadIdx.x] = total ? atomicAdd(reinterpret_cast<uint32_t*>(&result[2u + threadIdx.x]), total) : 0u;
    }
    __syncthreads();
    if (medium || large) {
        const uint32_t x = large ? 1u : 0u;
        uint32_t at = s_base[x];
        for (uint32_t w = 0; w < wid; ++w) at += s_cnt[x][w];
        at += (uint32_t)__popcll(votes[x] & ((1ull << lane) - 1ull));
        (large ? list_large : list_medium)[at] = c;
    }
}

// Kernels only, nothing waited for: the lists of the two larger instances are made on the
// device and walked by fixed grids.  Returns a HIP error code (0: fine).
int launch_inflate(shifter_ctx* ctx, const uint8_t* d_stream, uint64_t stream_bytes,
                   const uint64_t* d_seg_off, const uint16_t* d_sub_bits, const uint64_t* d_sub_marks,
                   uint64_t n_bytes, uint32_t n_chunks, uint8_t* d_out) {
    hipError_t e0 = codec_ensure_list(ctx, 2ull * n_chunks);
    if (e0 != hipSuccess) return (int)e0;
    uint32_t* list_medium = ctx->d_codec_list;
    uint32_t* list_large = ctx->d_codec_list + n_chunks;
    const uint32_t* n_medium = reinterpret_cast<const uint32_t*>(ctx->d_codec + 2);
    const uint32_t* n_large = reinterpret_cast<const uint32_t*>(ctx->d_codec + 3);
    codec_begin(ctx);
    {
        ProfileScope ps(ctx, K_INFLATE_CHUNK);
        codec_classify_kernel<<<(n_chunks + CLASSIFY_THREADS - 1) / CLASSIFY_THREADS, CLASSIFY_THREADS, 0, ctx->stream>>>(
            stream_bytes, d_seg_off, d_sub_bits, n_chunks, list_medium, list_large, ctx->d_codec);
        const uint32_t loop_grid = std::min(n_chunks, CODEC_LOOP_GRID);
        // the long segments first: their blocks run longest
        inflate_chunk_kernel<CODEC_SEG_LARGE, CODEC_SEG_MEDIUM + 1><<<loop_grid, CODEC_THREADS, 0, ctx->stream>>>(
            d_stream, stream_bytes, d_seg_off, d_sub_bits, d_sub_marks, n_bytes, n_chunks, d_out, ctx->d_codec,
            list_large, n_large);
        inflate_chunk_kernel<CODEC_SEG_MEDIUM, CODEC_SEG_SMALL + 1><<<loop_grid, CODEC_THREADS, 0, ctx->stream>>>(
            d_stream, stream_bytes, d_seg_off, d_sub_bits, d_sub_marks, n_bytes, n_chunks, d_out, ctx->d_codec,
            list_medium, n_medium);
        inflate_chunk_kernel<CODEC_SEG_SMALL, 0><<<n_chunks, CODEC_THREADS, 0, ctx->stream>>>(
            d_stream, stream_bytes, d_seg_off, d_sub_bits, d_sub_marks, n_bytes, n_chunks, d_out, ctx->d_codec,
            nullptr, nullptr);
    }
    codec_end(ctx);
    return 0;
}

}  // namespace shifter
