"""Pins for the codec oracle (Sec. III-E, Modules 7 and 8; RFC 1951).  CPU only.

The decoder is checked against the zlib library on streams of every block type and on
streams packed by hand from the RFC's code tables; the encoder's streams are inflated by
zlib (an independent decoder), its sizes follow closed forms, and small outputs are
compared with streams packed by hand.
"""
import zlib

import numpy as np
import pytest

from oracle import deflate_oracle as D


def pack(bit_string: str) -> bytes:
    """Bits in stream order ('0'/'1', blanks ignored) -> bytes, first bit = bit 0 of byte 0."""
    bits = [int(c) for c in bit_string if c in "01"]
    out = bytearray((len(bits) + 7) // 8)
    for i, b in enumerate(bits):
        out[i >> 3] |= b << (i & 7)
    return bytes(out)


def zinflate(raw: bytes) -> bytes:
    d = zlib.decompressobj(-15)
    out = d.decompress(raw)
    assert d.eof and d.unused_data == b""
    return out


def sparse_floats(n_floats, sparsity, seed):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(n_floats).astype(np.float32)
    w[rng.random(n_floats) < sparsity] = 0.0
    return w.tobytes()


def samples():
    rng = np.random.default_rng(0)
    yield b""
    yield b"a"
    yield b"abc" * 100
    yield bytes(1000)
    yield rng.integers(0, 256, 5000, dtype=np.uint8).tobytes()
    yield rng.integers(0, 4, 20000, dtype=np.uint8).tobytes()
    yield sparse_floats(6000, 0.9, 1)
    yield (b"the quick brown fox jumps over the lazy dog " * 300)[:70000]


# ----------------------------------------------------------------------------- decoder
@pytest.mark.parametrize("level,strategy", [(0, zlib.Z_DEFAULT_STRATEGY), (1, zlib.Z_DEFAULT_STRATEGY),
                                            (6, zlib.Z_DEFAULT_STRATEGY), (9, zlib.Z_DEFAULT_STRATEGY),
                                            (6, zlib.Z_FIXED), (6, zlib.Z_HUFFMAN_ONLY),
                                            (6, zlib.Z_RLE)])
def test_inflate_agrees_with_zlib_on_every_block_type(level, strategy):
    for data in samples():
        c = zlib.compressobj(level, zlib.DEFLATED, -15, 9, strategy)
        raw = c.compress(data) + c.flush()
        out, used = D.inflate(raw)
        assert out == data and used == len(raw)
        out, used = D.inflate(raw + b"trailing")           # stops at the final block
        assert out == data and used == len(raw)


def test_inflate_on_hand_packed_streams():
    # stored block: BFINAL=1, BTYPE=00, padding, LEN=3, NLEN=~3, "abc"
    assert D.inflate(bytes.fromhex("010300fcff616263")) == (b"abc", 8)
    # fixed block: header 1 10; 'a' = 0x30 + 97 = 10010001 (8 bits); end of block 0000000
    raw = pack("1 10 10010001 0000000")
    assert raw == bytes.fromhex("4b0400")
    assert D.inflate(raw) == (b"a", 3) and zinflate(raw) == b"a"
    # 'a', then length 4 (code 258 = 0000010) at distance 1 (code 00000): "aaaaa"
    raw = pack("1 10 10010001 0000010 00000 0000000")
    assert raw == bytes.fromhex("4b040100")
    assert D.inflate(raw) == (b"aaaaa", 4) and zinflate(raw) == b"aaaaa"
    # length 13 = code 266 (0001010) + extra bit 0; 14 = the same code + extra bit 1
    for extra, n in (("0", 13), ("1", 14)):
        raw = pack("1 10 10010001 0001010 " + extra + " 00000 0000000")
        assert D.inflate(raw)[0] == b"a" * (n + 1) == zinflate(raw)
    # literal 200 = 110010000 + 56 = 111001000 (9 bits); length 258 = code 285 = 11000101
    raw = pack("1 10 111001000 11000101 00000 0000000")
    assert D.inflate(raw)[0] == bytes([200]) * 259 == zinflate(raw)
    # distance 4 (code 3 = 00011): "abcd" + 6 bytes copied from 4 back
    lit = lambda ch: format(0x30 + ord(ch), "08b")
    raw = pack("1 10 " + " ".join(lit(c) for c in "abcd") + " 0000100 00011 0000000")
    assert D.inflate(raw)[0] == b"abcdabcdab" == zinflate(raw)
    # two blocks: a non-final empty stored block, then the final fixed block
    raw = pack("0 00 00000") + bytes.fromhex("0000ffff") + pack("1 10 10010001 0000000")
    assert D.inflate(raw)[0] == b"a" == zinflate(raw)


def test_inflate_rejects_broken_streams():
    with pytest.raises(ValueError):
        D.inflate(bytes.fromhex("010300fcfe616263"))          # NLEN is not ~LEN
    with pytest.raises(ValueError):
        D.inflate(bytes.fromhex("010300fcff6162"))            # truncated stored block
    with pytest.raises(ValueError):
        D.inflate(pack("1 11"))                               # reserved block type
    with pytest.raises(ValueError):
        D.inflate(pack("1 10 0000010 00000 0000000"))         # match before any output
    with pytest.raises(ValueError):
        D.inflate(pack("1 10 10010001"))                      # no end of block


# ----------------------------------------------------------------------------- encoder
def test_run_pieces_rule():
    assert D.run_pieces(3) == [3] and D.run_pieces(258) == [258]
    assert D.run_pieces(259) == [256, 3] and D.run_pieces(260) == [257, 3]
    assert D.run_pieces(261) == [258, 3] and D.run_pieces(511) == [258, 253]
    assert D.run_pieces(516) == [258, 258] and D.run_pieces(517) == [258, 256, 3]
    for r in range(3, 1500):
        p = D.run_pieces(r)
        assert sum(p) == r and all(3 <= x <= 258 for x in p)


def test_tokenize_sub_rule():
    assert D.tokenize_sub(b"") == []
    assert D.tokenize_sub(b"abc") == [(0, 97), (0, 98), (0, 99)]
    assert D.tokenize_sub(b"aaa") == [(0, 97)] * 3                  # runs of 3 stay literals
    assert D.tokenize_sub(b"aaaa") == [(0, 97), (1, 3)]
    assert D.tokenize_sub(b"xaaaaay") == [(0, 120), (0, 97), (1, 4), (0, 121)]
    assert D.tokenize_sub(bytes(512)) == [(0, 0), (1, 258), (1, 253)]
    assert D.tokenize_sub(bytes(5) + b"\1" * 4) == [(0, 0), (1, 4), (0, 1), (1, 3)]


def encoder_inputs():
    rng = np.random.default_rng(5)
    C, S = D.CHUNK, D.SUB
    for n in (0, 1, 3, 4, 5, S - 1, S, S + 1, C - 1, C, C + 1):
        yield bytes(n)
        yield rng.integers(0, 256, n, dtype=np.uint8).tobytes()
    yield sparse_floats(3 * C // 4 + 123, 0.5, 2)
    yield sparse_floats(3 * C // 4 + 77, 0.9, 3)
    yield sparse_floats(C // 2 + 5, 0.99, 4)
    for run in (259, 260, 261, 262, 263, 264, 265, 511, 512, 513, 516, 517, 2 * C + 9):
        yield b"ab" + b"\7" * run + b"cd"                # runs across sub-chunks and chunks
        yield b"x" * (S - 130) + bytes(run) + b"\xff" * 700
    yield bytes(range(256)) * 300                         # nothing repeats: stored segments
    noise = rng.integers(0, 256, 4 * C, dtype=np.uint8).tobytes()
    # coded and stored sub-chunks in one segment, in every order
    yield bytes(S) + noise[:S] + bytes(3 * S) + noise[S:3 * S] + bytes(100)
    yield noise[:S] + bytes(S) + noise[S:2 * S + 7] + bytes(2 * S - 7) + noise[:S // 2]
    yield noise[:3 * S] + bytes(C - 3 * S) + bytes(C - S) + noise[:S] + noise[:S] + bytes(77)
    yield sparse_floats(C // 4, 0.9, 8) + noise[:C // 2] + sparse_floats(C // 4 + 31, 0.6, 9)
    yield (b"\0\0\0\0\x12\x34\x56\x3f" * 9000)[:2 * C + 4000]


def expected_segment_bytes(side, sub_lens):
    """Length of a sub-chunk-built segment from its side information: the same walk as
    the encoder's, on bit counts only."""
    pos, in_block = 0, False
    for v, n in zip(side, sub_lens):
        if n == 0:
            assert v == 0
            continue
        if v == D.STORED_MARK:
            pos += (7 if in_block else 0) + 3
            pos = (pos + 7) // 8 * 8 + 32 + 8 * n
            in_block = False
        else:
            pos += (0 if in_block else 3) + v
            in_block = True
    pos += (7 if in_block else 0) + 3
    return (pos + 7) // 8 + 4


def test_encoder_output_inflates_with_zlib_and_sizes_add_up():
    nsub = D.CHUNK // D.SUB
    mixed = 0
    for data in encoder_inputs():
        stream, seg_off, side = D.deflate_runs(data)
        assert zinflate(stream) == data
        n_chunks = max(1, -(-len(data) // D.CHUNK))
        assert len(seg_off) == n_chunks + 1 and seg_off[0] == 0 and seg_off[-1] == len(stream)
        assert len(side) == n_chunks * nsub
        for c in range(n_chunks):
            seg = stream[seg_off[c]:seg_off[c + 1]]
            chunk = data[c * D.CHUNK:(c + 1) * D.CHUNK]
            d = zlib.decompressobj(-15)                   # every segment stands alone
            assert d.decompress(seg) == chunk and d.unused_data == b""
            assert d.eof == (c == n_chunks - 1)
            here = side[c * nsub:(c + 1) * nsub]
            sub_lens = [len(chunk[s * D.SUB:(s + 1) * D.SUB]) for s in range(nsub)]
            if not any(here):                             # the whole chunk in one stored block
                assert len(seg) == len(chunk) + 5 and (seg[0] >> 1) & 3 == 0
            else:
                assert len(seg) == expected_segment_bytes(here, sub_lens) < len(chunk) + 5
                assert seg[-4:] == b"\x00\x00\xff\xff"
                for v, n, s in zip(here, sub_lens, range(nsub)):
                    toks = D.tokenize_sub(chunk[s * D.SUB:(s + 1) * D.SUB])
                    t = D.token_bits(toks)
                    assert v == (D.STORED_MARK if t > 8 * n + D.STORED_MARGIN else t)
                mixed += D.STORED_MARK in here and any(0 < v < D.STORED_MARK for v in here)
        if len(data) <= 3000:
            assert D.inflate(stream) == (data, len(stream))
    assert mixed >= 3                                     # segments with both kinds occur


def test_encoder_closed_forms_and_hand_packed_streams():
    assert D.deflate_runs(b"") == (bytes.fromhex("010000ffff"), [0, 5], [0] * 64)
    # five zero bytes: literal 0 (00110000), length 4, end of block, final empty stored block
    stream, seg_off, sub_bits = D.deflate_runs(bytes(5))
    assert stream == pack("0 10 00110000 0000010 00000 0000000 1 00") + bytes.fromhex("0000ffff")
    assert sub_bits[:2] == [20, 0] and seg_off == [0, 9]
    # 512 zeros, then 60 bytes that take 9 bits each: a coded and a stored sub-chunk.
    # 253 = code 284 (11000100) with extra bits 26, least significant first: 01011
    tail = bytes([200, 201] * 30)
    stream, seg_off, side = D.deflate_runs(bytes(512) + tail)
    assert side[:3] == [39, D.STORED_MARK, 0]
    assert stream == (pack("0 10 00110000 11000101 00000 11000100 01011 00000 0000000 0 00")
                      + bytes.fromhex("3c00c3ff") + tail + bytes.fromhex("010000ffff"))
    assert len(pack("0 10 00110000 11000101 00000 11000100 01011 00000 0000000 0 00")) == 7
    # alone, the same 60 bytes are one stored block: the sub-chunk form would be longer
    assert D.deflate_runs(tail)[0] == bytes.fromhex("013c00c3ff") + tail
    # four bytes would take 9 bytes as a Huffman segment, and take 9 stored: stored wins ties
    assert D.deflate_runs(b"abcd")[0] == bytes.fromhex("010400fbff") + b"abcd"
    # a chunk of zeros: per sub-chunk literal (8) + 258 (8 + 5) + 253 (8 + 5 extra + 5) bits
    stream, seg_off, sub_bits = D.deflate_runs(bytes(D.CHUNK))
    assert sub_bits == [39] * 64 and len(stream) == (3 + 64 * 39 + 7 + 3 + 7) // 8 + 4 == 318
    # two chunks: the first segment ends with a non-final empty stored block
    stream, seg_off, _ = D.deflate_runs(bytes(D.CHUNK + 8))
    assert seg_off == [0, 318, 318 + 9]
    first_tail = stream[seg_off[1] - 5] >> ((3 + 64 * 39 + 7) % 8)
    assert first_tail & 7 == 0                            # BFINAL=0, BTYPE=00
    # random bytes: stored, 5 bytes per chunk
    data = np.random.default_rng(1).integers(0, 256, 2 * D.CHUNK + 10, dtype=np.uint8).tobytes()
    stream, seg_off, sub_bits = D.deflate_runs(data)
    assert seg_off == [0, D.CHUNK + 5, 2 * D.CHUNK + 10, 2 * D.CHUNK + 25] and not any(sub_bits)
    assert stream[:5] == bytes.fromhex("000080ff7f") and stream[5:5 + D.CHUNK] == data[:D.CHUNK]
    # a sparse model compresses by about the share of zeros
    data = sparse_floats(40000, 0.95, 7)
    stream, _, _ = D.deflate_runs(data)
    assert 8 < len(data) / len(stream) < 20


@pytest.mark.parametrize("mistake", ["code_bit_order", "nlen", "length_base", "extra_bits",
                                     "run_of_three_as_match", "literal_9bit"])
def test_planted_encoder_mistakes_are_caught(mistake, monkeypatch):
    data = (b"ab" + bytes(300) + bytes([200]) * 20 + bytes(range(256)) + bytes(17) + b"\x09" * 13
            + b"zz" * 700)
    assert zinflate(D.deflate_runs(data)[0]) == data
    if mistake == "code_bit_order":
        monkeypatch.setattr(D._BitWriter, "code", lambda self, c, n: self.bits(c, n))
    elif mistake == "nlen":
        real = D._BitWriter.bits
        monkeypatch.setattr(D._BitWriter, "bits",
                            lambda self, v, n: real(self, 0 if (v, n) == (0xFFFF, 16) else v, n))
    elif mistake == "length_base":
        monkeypatch.setattr(D, "LENGTH_BASE", D.LENGTH_BASE[:8] + [12] + D.LENGTH_BASE[9:])
    elif mistake == "extra_bits":
        monkeypatch.setattr(D, "LENGTH_EXTRA", [0] * 29)
    elif mistake == "run_of_three_as_match":
        monkeypatch.setattr(D, "run_pieces", lambda r: [r + 1])
    elif mistake == "literal_9bit":
        real_lit = D._fixed_literal
        monkeypatch.setattr(D, "_fixed_literal",
                            lambda w, v: w.code(0b110000000 + (v - 144), 9) if 144 <= v < 256
                            else real_lit(w, v))
    try:
        ok = zinflate(D.deflate_runs(data)[0]) == data
    except (zlib.error, AssertionError):
        ok = False
    assert not ok


# ----------------------------------------------------------------------------- quarter marks
def sub_bit_starts(side, sub_lens):
    """Bit position, inside its segment, of the first token of every coded sub-chunk (the
    layout rule of the segment written out once more, from the side information alone)."""
    pos, in_block, starts = 0, False, []
    for v, n in zip(side, sub_lens):
        if n == 0:
            starts.append(None)
            continue
        if v == D.STORED_MARK:
            starts.append(None)
            pos += (7 if in_block else 0) + 3
            pos = (pos + 7) // 8 * 8 + 32 + 8 * n
            in_block = False
        else:
            pos += 0 if in_block else 3
            starts.append(pos)
            pos += v
            in_block = True
    return starts


def decode_quarter(seg: bytes, bit: int, bit_end: int, first_byte_known=None):
    """Tokens from bit to bit_end with the decoder's own primitives: returns the bytes they
    produce; the first token must be a literal."""
    br = D._Bits(seg)
    br.pos = bit
    out = bytearray()
    while br.pos < bit_end:
        sym = D._symbol(br, D.FIXED_LIT)
        if sym < 256:
            out.append(sym)
        else:
            assert 257 <= sym <= 285 and out, "a quarter starts with a literal"
            ln = D.LENGTH_BASE[sym - 257] + br.bits(D.LENGTH_EXTRA[sym - 257])
            assert D._symbol(br, D.FIXED_DIST) == 0
            out += bytes([out[-1]]) * ln
    assert br.pos == bit_end
    return bytes(out)


def test_quarter_marks_by_hand():
    f = lambda fields: sum((d | (o << 11)) << (20 * q) for q, (d, o) in enumerate(fields))
    # 512 zeros: one literal and two matches, 39 bits, nothing starts after offset 0
    assert D.quarter_marks(bytes(512)) == f([(39, 384), (0, 256), (0, 128)])
    # 512 bytes without runs, all below 144: 8 bits each, a literal at every boundary
    assert D.quarter_marks(bytes(i % 100 for i in range(512))) == f([(1024, 0)] * 3)
    # ... all 9-bit literals
    assert D.quarter_marks(bytes(200 + i % 50 for i in range(512))) == f([(1152, 0)] * 3)
    # a run across the first boundary: 120 literals (8 bits), then 20 zeros from offset 120
    # (literal 8 bits + length 19 = code 269 with 2 extra bits, 7 + 2 + 5 = 14 bits), then
    # literals; the second decoder starts at offset 140, after 120 * 8 + 22 bits
    sub = bytes(1 + i % 100 for i in range(120)) + bytes(20) + bytes(1 + i % 100 for i in range(372))
    assert D.quarter_marks(sub) == f([(120 * 8 + 22, 12), ((256 - 140) * 8, 0), (1024, 0)])
    # a short sub-chunk: 130 bytes, boundaries 128, 130, 130
    sub = bytes(1 + i % 100 for i in range(130))
    assert D.quarter_marks(sub) == f([(1024, 0), (16, 0), (0, 0)])
    # 300 bytes ending in a run that covers two boundaries
    sub = bytes(1 + i % 100 for i in range(100)) + bytes([7]) * 200
    assert D.tokenize_sub(sub)[100:] == [(0, 7), (1, 199)]
    # literal 7: 8 bits; length 199 = code 283 (base 195, 5 extra bits): 8 + 5 + 5 = 18 bits
    assert D.quarter_marks(sub) == f([(100 * 8 + 26, 300 - 128), (0, 300 - 256), (0, 0)])


def test_every_quarter_decodes_alone_from_its_mark():
    nsub = D.CHUNK // D.SUB
    checked = 0
    for data in encoder_inputs():
        stream, seg_off, side = D.deflate_runs(data)
        marks = D.deflate_marks(data, side)
        assert len(marks) == len(side)
        for c in range(len(seg_off) - 1):
            seg = stream[seg_off[c]:seg_off[c + 1]]
            chunk = data[c * D.CHUNK:(c + 1) * D.CHUNK]
            here = side[c * nsub:(c + 1) * nsub]
            sub_lens = [len(chunk[s * D.SUB:(s + 1) * D.SUB]) for s in range(nsub)]
            if not any(here):
                assert not any(marks[c * nsub:(c + 1) * nsub])
                continue
            for s, (start, v, n) in enumerate(zip(sub_bit_starts(here, sub_lens), here, sub_lens)):
                mark = marks[c * nsub + s]
                if start is None:
                    assert mark == 0
                    continue
                sub = chunk[s * D.SUB:(s + 1) * D.SUB]
                bits, offs = [0], [0]
                for q in (1, 2, 3):
                    field = (mark >> (20 * (q - 1))) & 0xFFFFF
                    bits.append(bits[-1] + (field & 0x7FF))
                    offs.append(min(D.QUARTER * q, n) + (field >> 11))
                bits.append(v)
                offs.append(n)
                assert mark >> 60 == 0 and offs == sorted(offs) and bits == sorted(bits)
                for q in range(4):
                    got = decode_quarter(seg, start + bits[q], start + bits[q + 1])
                    assert got == sub[offs[q]:offs[q + 1]]
                    # the first literal at or after the boundary, not a later one
                    assert q == 0 or offs[q] == min(D.QUARTER * q, n) or \
                        len(set(sub[min(D.QUARTER * q, n) - 1:offs[q]])) == 1
                    checked += 1
    assert checked > 2000


def test_planted_mark_mistakes_are_caught(monkeypatch):
    sub = bytes(1 + i % 100 for i in range(120)) + bytes(20) + bytes(1 + i % 100 for i in range(372))
    good = D.quarter_marks(sub)
    real = D.tokenize_sub
    # matches counted with the wrong literal: the run's match left to the next decoder
    monkeypatch.setattr(D, "token_bits", lambda toks: 0 if toks and toks[0][0] == 1 else
                        8 * len(toks))
    assert D.quarter_marks(sub) != good
    monkeypatch.undo()
    assert D.quarter_marks(sub) == good
