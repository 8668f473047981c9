"""CPU oracle for the portfolio codec.  TEST INFRASTRUCTURE ONLY.

Plain, slow Python written from the format definition; it shares no code with the HIP
library and must never be imported by the product path: only the tests, the smoke check
and the benchmark's CPU-baseline leg call it.

Phase 3 of the paper (Sec. III-E: Module 7 deflates the portfolio, Module 8 inflates the
model that is to run) stores inactive models as DEFLATE streams (RFC 1951), which pays
because the zero weights of sparse models repeat.  Two things are defined here:

* ``inflate``  - a DEFLATE decoder following RFC 1951 section 3.2 step by step (stored,
  fixed-Huffman and dynamic-Huffman blocks, distances up to 32 KiB).  It is the meaning
  of a stream: whatever an encoder emits is correct iff it inflates to the input.
* ``deflate_runs`` - the one encoder the library implements, stated as a deterministic
  rule so that its output can be compared bit for bit.  DEFLATE leaves the choice of
  blocks and matches to the encoder; this one is built for chunk-parallel decoding:

  - the input is cut into chunks of CHUNK = 32768 bytes, each chunk into sub-chunks of
    SUB = 512 bytes; every chunk becomes a byte-aligned *segment*, and the stream is the
    segments in order;
  - inside a sub-chunk, left to right: a maximal run of r >= 4 equal bytes (cut at the
    sub-chunk's end) is one literal followed by matches of distance 1 that cover the other
    R = r - 1 bytes: pieces of 258 while more than 260 bytes remain, then one piece if at
    most 258 remain, else the two pieces (remaining - 3, 3); everything else is literals;
  - a sub-chunk whose tokens take more than 8 * (its bytes) + STORED_MARGIN bits is
    *stored*: it becomes a stored block of its own (its bytes verbatim), which is both
    shorter and copied rather than decoded; the others are *coded*;
  - a segment is built sub-chunk by sub-chunk (empty ones are skipped): a coded sub-chunk
    opens a fixed-Huffman block (BFINAL=0, BTYPE=01) unless one is open, and appends its
    tokens; a stored sub-chunk closes the open block with end-of-block, then is a stored
    block (BFINAL=0, BTYPE=00, padding to a byte, LEN, NLEN, the bytes); after the last
    sub-chunk the open block is closed, and an empty stored block (header, padding, LEN=0,
    NLEN=0xFFFF) re-aligns the stream and carries BFINAL=1 in the last segment;
  - if that is not shorter than one stored block holding the whole chunk (m + 5 bytes),
    the segment is that stored block instead (BFINAL=1 in the last segment); an empty
    input is the single segment 01 00 00 FF FF;
  - side information for parallel decoding (not part of the DEFLATE stream): the byte
    offset of every segment, and per sub-chunk the number of token bits if it is coded,
    0xFFFF if it is stored (all 0 when the whole chunk is one stored block);
  - more side information, so that four decoders can share a coded sub-chunk of n bytes
    (``quarter_marks``): for q = 1, 2, 3 let B_q = min(128 q, n), o_q the offset of the first
    literal token at or after B_q (n if there is none) and b_q the bits of all tokens
    before that literal (a run's matches go with the literal that starts it; all the
    sub-chunk's token bits if there is none), b_0 = 0.  The mark of the sub-chunk is the
    integer sum over q of ((b_q - b_(q-1)) + ((o_q - B_q) << 11)) << (20 (q - 1)); stored
    and empty sub-chunks, and chunks that are one stored block, have mark 0.  Decoder q
    starts at bit b_q and offset o_q and stops at b_(q+1), o_(q+1).

All are pinned by tests that do not go through them: ``inflate`` against the zlib
library on streams of every block type and against streams assembled by hand from the
RFC's tables; ``deflate_runs`` by inflating its output with zlib, by closed forms for
its sizes, and by hand-assembled expected streams; ``quarter_marks`` by hand-worked
marks, and by decoding every quarter of the encoder's streams on its own, from its mark
alone, with the decoder's primitives.  None is "parity unpinned".
"""
from __future__ import annotations

from typing import List, Tuple

CHUNK = 32768
SUB = 512
STORED_MARGIN = 48
STORED_MARK = 0xFFFF
QUARTER = 128                 # bytes of a sub-chunk per decoder

# RFC 1951 section 3.2.5: base length and number of extra bits of length codes 257..285
LENGTH_BASE = [3, 4, 5, 6, 7, 8, 9, 10, 11, 13, 15, 17, 19, 23, 27, 31, 35, 43, 51, 59, 67, 83,
               99, 115, 131, 163, 195, 227, 258]
LENGTH_EXTRA = [0, 0, 0, 0, 0, 0, 0, 0, 1, 1, 1, 1, 2, 2, 2, 2, 3, 3, 3, 3, 4, 4, 4, 4, 5, 5,
                5, 5, 0]
# base distance and extra bits of distance codes 0..29
DIST_BASE = [1, 2, 3, 4, 5, 7, 9, 13, 17, 25, 33, 49, 65, 97, 129, 193, 257, 385, 513, 769,
             1025, 1537, 2049, 3073, 4097, 6145, 8193, 12289, 16385, 24577]
DIST_EXTRA = [0, 0, 0, 0, 1, 1, 2, 2, 3, 3, 4, 4, 5, 5, 6, 6, 7, 7, 8, 8, 9, 9, 10, 10, 11, 11,
              12, 12, 13, 13]
# order in which code-length-code lengths are sent (section 3.2.7)
CL_ORDER = [16, 17, 18, 0, 8, 7, 9, 6, 10, 5, 11, 4, 12, 3, 13, 2, 14, 1, 15]


# ----------------------------------------------------------------------------- decoder
class _Bits:
    """Bit reader: data elements start at the least significant bit of each byte."""
    def __init__(self, data: bytes):
        self.data, self.pos = data, 0            # pos in bits

    def bit(self) -> int:
        if self.pos >> 3 >= len(self.data):
            raise ValueError("stream ends inside a block")
        b = (self.data[self.pos >> 3] >> (self.pos & 7)) & 1
        self.pos += 1
        return b

    def bits(self, n: int) -> int:               # n-bit integer, least significant bit first
        v = 0
        for i in range(n):
            v |= self.bit() << i
        return v

    def align(self) -> None:
        self.pos = (self.pos + 7) & ~7


def _canonical(lengths: List[int]) -> dict:
    """Section 3.2.2: codes of one length are consecutive values in symbol order, and
    shorter codes precede longer ones.  Returns {(length, code): symbol}."""
    max_len = max(lengths) if lengths else 0
    count = [0] * (max_len + 1)
    for l in lengths:
        if l:
            count[l] += 1
    code, next_code = 0, [0] * (max_len + 2)
    for l in range(1, max_len + 1):
        code = (code + count[l - 1]) << 1
        next_code[l] = code
    table = {}
    for sym, l in enumerate(lengths):
        if l:
            table[(l, next_code[l])] = sym
            next_code[l] += 1
    return table


def _symbol(br: _Bits, table: dict) -> int:
    code = 0
    for l in range(1, 16):                       # Huffman codes arrive most significant bit first
        code = (code << 1) | br.bit()
        if (l, code) in table:
            return table[(l, code)]
    raise ValueError("invalid Huffman code")


FIXED_LIT = _canonical([8] * 144 + [9] * 112 + [7] * 24 + [8] * 8)
FIXED_DIST = _canonical([5] * 30)


def inflate(data: bytes) -> Tuple[bytes, int]:
    """RFC 1951 section 3.2.3: decodes blocks until one with BFINAL set.
    Returns (output, number of input bytes consumed)."""
    br, out = _Bits(data), bytearray()
    while True:
        final, btype = br.bit(), br.bits(2)
        if btype == 0:
            br.align()
            ln, nln = br.bits(16), br.bits(16)
            if ln ^ nln != 0xFFFF:
                raise ValueError("stored block: LEN and NLEN disagree")
            start = br.pos >> 3
            if start + ln > len(data):
                raise ValueError("stream ends inside a stored block")
            out += data[start:start + ln]
            br.pos += 8 * ln
        elif btype in (1, 2):
            if btype == 1:
                lit, dist = FIXED_LIT, FIXED_DIST
            else:
                hlit, hdist, hclen = br.bits(5) + 257, br.bits(5) + 1, br.bits(4) + 4
                cl = [0] * 19
                for i in range(hclen):
                    cl[CL_ORDER[i]] = br.bits(3)
                cl_table = _canonical(cl)
                lens: List[int] = []
                while len(lens) < hlit + hdist:
                    s = _symbol(br, cl_table)
                    if s < 16:
                        lens.append(s)
                    elif s == 16:
                        if not lens:
                            raise ValueError("repeat with no previous length")
                        lens += [lens[-1]] * (3 + br.bits(2))
                    elif s == 17:
                        lens += [0] * (3 + br.bits(3))
                    else:
                        lens += [0] * (11 + br.bits(7))
                if len(lens) != hlit + hdist:
                    raise ValueError("code lengths overrun")
                lit, dist = _canonical(lens[:hlit]), _canonical(lens[hlit:])
            while True:
                s = _symbol(br, lit)
                if s < 256:
                    out.append(s)
                elif s == 256:
                    break
                else:
                    if s > 285:
                        raise ValueError("invalid length code")
                    ln = LENGTH_BASE[s - 257] + br.bits(LENGTH_EXTRA[s - 257])
                    d = _symbol(br, dist)
                    if d > 29:
                        raise ValueError("invalid distance code")
                    d = DIST_BASE[d] + br.bits(DIST_EXTRA[d])
                    if d > len(out):
                        raise ValueError("distance reaches before the start")
                    for _ in range(ln):          # may overlap itself: byte by byte
                        out.append(out[-d])
        else:
            raise ValueError("reserved block type")
        if final:
            return bytes(out), (br.pos + 7) >> 3


# ----------------------------------------------------------------------------- encoder
class _BitWriter:
    def __init__(self):
        self.out, self.acc, self.n = bytearray(), 0, 0

    def bits(self, v: int, n: int) -> None:      # integer, least significant bit first
        self.acc |= v << self.n
        self.n += n
        while self.n >= 8:
            self.out.append(self.acc & 0xFF)
            self.acc >>= 8
            self.n -= 8

    def code(self, c: int, n: int) -> None:      # Huffman code, most significant bit first
        for i in range(n - 1, -1, -1):
            self.bits((c >> i) & 1, 1)

    def align(self) -> None:
        if self.n:
            self.bits(0, 8 - self.n)


def _fixed_literal(w: _BitWriter, v: int) -> None:
    """Section 3.2.6: literal/length value -> fixed code."""
    if v < 144:
        w.code(0b00110000 + v, 8)
    elif v < 256:
        w.code(0b110010000 + (v - 144), 9)
    elif v < 280:
        w.code(v - 256, 7)
    else:
        w.code(0b11000000 + (v - 280), 8)


def _fixed_match(w: _BitWriter, length: int) -> None:
    """A match of distance 1: length code, its extra bits, the 5-bit distance code 0."""
    idx = max(i for i in range(29) if LENGTH_BASE[i] <= length)
    _fixed_literal(w, 257 + idx)
    w.bits(length - LENGTH_BASE[idx], LENGTH_EXTRA[idx])
    w.code(0, 5)


def run_pieces(r_rest: int) -> List[int]:
    """Match lengths covering the R = r - 1 bytes that follow a run's first byte."""
    assert r_rest >= 3
    pieces = []
    while r_rest > 260:
        pieces.append(258)
        r_rest -= 258
    if r_rest <= 258:
        pieces.append(r_rest)
    else:
        pieces += [r_rest - 3, 3]
    return pieces


def tokenize_sub(b: bytes) -> List[Tuple[int, int]]:
    """Tokens of one sub-chunk: (0, byte) literals and (1, length) distance-1 matches."""
    toks, i, n = [], 0, len(b)
    while i < n:
        r = 1
        while i + r < n and b[i + r] == b[i]:
            r += 1
        if r >= 4:
            toks.append((0, b[i]))
            toks += [(1, p) for p in run_pieces(r - 1)]
            i += r
        else:
            toks.append((0, b[i]))
            i += 1
    return toks


def _emit_tokens(w: _BitWriter, toks) -> None:
    for kind, val in toks:
        if kind == 0:
            _fixed_literal(w, val)
        else:
            _fixed_match(w, val)


def token_bits(toks) -> int:
    w = _BitWriter()
    _emit_tokens(w, toks)
    return 8 * len(w.out) + w.n


def deflate_runs(data: bytes) -> Tuple[bytes, List[int], List[int]]:
    """Returns (stream, segment byte offsets [n_chunks + 1], side information per sub-chunk
    [n_chunks * (CHUNK // SUB)])."""
    n = len(data)
    n_chunks = max(1, (n + CHUNK - 1) // CHUNK)
    nsub = CHUNK // SUB
    stream, seg_off, side = bytearray(), [0], []
    for c in range(n_chunks):
        chunk = data[c * CHUNK:(c + 1) * CHUNK]
        m = len(chunk)
        last = 1 if c == n_chunks - 1 else 0
        w = _BitWriter()
        in_block = False
        side_here = []
        for s in range(nsub):
            sub = chunk[s * SUB:(s + 1) * SUB]
            if not sub:
                side_here.append(0)
                continue
            toks = tokenize_sub(sub)
            t_bits = token_bits(toks)
            if t_bits > 8 * len(sub) + STORED_MARGIN:
                if in_block:
                    _fixed_literal(w, 256)
                    in_block = False
                w.bits(0, 1)
                w.bits(0, 2)
                w.align()
                w.bits(len(sub), 16)
                w.bits(len(sub) ^ 0xFFFF, 16)
                for b in sub:
                    w.bits(b, 8)
                side_here.append(STORED_MARK)
            else:
                if not in_block:
                    w.bits(0, 1)
                    w.bits(1, 2)
                    in_block = True
                _emit_tokens(w, toks)
                side_here.append(t_bits)
        if in_block:
            _fixed_literal(w, 256)
        w.bits(last, 1)
        w.bits(0, 2)
        w.align()
        w.bits(0x0000, 16)
        w.bits(0xFFFF, 16)
        if m + 5 <= len(w.out):
            seg = bytes([last]) + m.to_bytes(2, "little") + (m ^ 0xFFFF).to_bytes(2, "little") \
                + chunk
            side_here = [0] * nsub
        else:
            seg = bytes(w.out)
        stream += seg
        seg_off.append(len(stream))
        side += side_here
    return bytes(stream), seg_off, side


def quarter_marks(sub: bytes) -> int:
    """The mark of a coded sub-chunk: where the decoders of its second, third and fourth
    128 bytes start (see the module's header)."""
    n = len(sub)
    lits, off, bit = [], 0, 0                    # (offset, bits before it) of every literal token
    for kind, val in tokenize_sub(sub):
        if kind == 0:
            lits.append((off, bit))
            off += 1
        else:
            off += val
        bit += token_bits([(kind, val)])
    mark, b_prev = 0, 0
    for q in (1, 2, 3):
        bound = min(QUARTER * q, n)
        o_q, b_q = next(((o, b) for o, b in lits if o >= bound), (n, bit))
        mark |= ((b_q - b_prev) | ((o_q - bound) << 11)) << (20 * (q - 1))
        b_prev = b_q
    return mark


def deflate_marks(data: bytes, side: List[int]) -> List[int]:
    """Marks of every sub-chunk of ``data``, given the side information ``deflate_runs``
    returned for it."""
    nsub = CHUNK // SUB
    marks = []
    for k, v in enumerate(side):
        c, s = divmod(k, nsub)
        sub = data[c * CHUNK + s * SUB:min(c * CHUNK + (s + 1) * SUB, (c + 1) * CHUNK)]
        marks.append(quarter_marks(sub) if v not in (0, STORED_MARK) else 0)
    return marks
