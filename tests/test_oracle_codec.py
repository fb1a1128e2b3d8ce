"""Pins of the swap-encoding oracle: hand-written examples of every slot mode, the inverse property on edge cases, an
independent bit-by-bit decoder, and structural invariants of the format."""
import numpy as np
import pytest

from oracle import swap_codec as C

SLOT = 4368          # 256 bitmap + 16 header + 2 * 2048 values


def test_hand_written_raw_example():
    # 16 elements: non-zeros at 1, 3, 4, 7 and 15 (-0.0 = 0x8000 and a NaN pattern count as non-zero); the exponent
    # fields 127, 0, 255, 0, 255 span more than 31: raw slot
    bits = np.array([0, 0x3F80, 0, 0x8000, 0x7FC1, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0, 0xFFFF], dtype=np.uint16)
    buf, defined = C.encode(bits)
    assert buf.size == SLOT + 16 + 16                       # one slot, counts padded to 16, trailer
    assert buf[0] == 0b10011010 and buf[1] == 0b10000000 and not buf[2:256].any()
    assert buf[256] == 0 and buf[257] == 0                  # mode raw
    assert list(buf[258:260]) == [10, 0]                    # value bytes
    assert list(buf[272:282]) == [0x80, 0x3F, 0x00, 0x80, 0xC1, 0x7F, 0x01, 0x00, 0xFF, 0xFF]
    assert list(buf[SLOT:SLOT + 4]) == [5, 0, 10, 0]        # count of the only slot, flags clear, 10 value bytes
    assert list(buf[SLOT + 16:SLOT + 24]) == [0x20, 0x01, 0, 0, 0, 0, 0, 0]    # 288 = 272 + 16, little-endian
    assert defined[:260].all() and not defined[260:272].any() and defined[272:282].all() and not defined[282:SLOT].any()
    assert defined[SLOT:SLOT + 4].all() and not defined[SLOT + 4:SLOT + 16].any()
    assert defined[SLOT + 16:SLOT + 24].all() and not defined[SLOT + 24:].any()
    assert np.array_equal(C.decode(buf, 16), bits)
    assert C.moved_bytes(buf, 16) == 272 + 16


def test_hand_written_packed_examples():
    # signed, narrow (12 bits): 1.0 (exponent 127), -0.5 (126, sign), 0x3E91 (125, mantissa 0x11), 0x4011 (128, mantissa
    # 0x11): emax = 128, codes sign << 11 | (emax - e) << 7 | mantissa = 0x080, 0x900, 0x191, 0x011; bit stream, low first:
    #   byte 0 = 0x80, byte 1 = 0x0 | 0x0 << 4, byte 2 = 0x90, byte 3 = 0x91, byte 4 = 0x1 | 0x1 << 4, byte 5 = 0x01
    bits = np.array([0, 0x3F80, 0, 0xBF00, 0x3E91, 0, 0, 0x4011] + [0] * 8, dtype=np.uint16)
    buf, defined = C.encode(bits)
    assert buf[0] == 0b10011010 and buf[1] == 0
    assert buf[256] == 1 + 4 and buf[257] == 128            # packed, signed
    assert list(buf[272:278]) == [0x80, 0x00, 0x90, 0x91, 0x11, 0x01]
    assert list(buf[258:260]) == [6, 0]
    assert list(buf[SLOT:SLOT + 4]) == [4, 0xA0, 6, 0]      # count 4, bit 15: packed, bit 13: signed; 6 value bytes
    assert defined[272:278].all() and not defined[278:SLOT].any()
    assert C.moved_bytes(buf, 16) == 272 + 16
    assert np.array_equal(C.decode(buf, 16), bits)
    # an odd count ends in half a byte whose unused high bits are zero.  The first three values alone have
    # emax = 127: codes 0x000, 0x880, 0x111 -> bytes 0x00, 0x0 | 0x0 << 4, 0x88, 0x11, 0x1
    odd, d = C.encode(np.array([0, 0x3F80, 0, 0xBF00, 0x3E91, 0, 0, 0], dtype=np.uint16))
    assert odd[257] == 127 and list(odd[272:277]) == [0x00, 0x00, 0x88, 0x11, 0x01]
    assert list(odd[SLOT:SLOT + 4]) == [3, 0xA0, 5, 0] and d[272:277].all() and not d[277:SLOT].any()

    # unsigned, narrow: the same magnitudes, all positive.  Packed they would be 4 codes of 11 bits = 6 bytes; split
    # they take 4 bytes and a unary stream, which is fewer: differences to emax = 128 are d = 1, 2, 3, 0; bytes
    # (d & 1) << 7 | mantissa = 0x80, 0x00, 0x91, 0x11; quotients d >> 1 = 0, 1, 1, 0 in unary, low bit first:
    # "1", "01", "01", "1" -> stream bits 1,0,1,0,1,1 = 0b110101 = 0x35: 5 value bytes
    pos = np.array([0, 0x3F80, 0, 0x3F00, 0x3E91, 0, 0, 0x4011] + [0] * 8, dtype=np.uint16)
    buf, defined = C.encode(pos)
    assert buf[256] == 1 + 8 and buf[257] == 128
    assert list(buf[272:277]) == [0x80, 0x00, 0x91, 0x11, 0x35]
    assert list(buf[258:260]) == [5, 0]
    assert list(buf[SLOT:SLOT + 4]) == [4, 0x90, 5, 0]      # bit 15: packed, bit 12: split
    assert defined[272:277].all() and not defined[277:SLOT].any()
    assert np.array_equal(C.decode(buf, 16), pos)
    assert C.moved_bytes(buf, 16) == 272 + 16
    # five elements with exponents 130, 130, 121, 130, 129 (d = 0, 0, 9, 0, 1): split would take 5 bytes padded to 8
    # and 5 + 4 unary bits = 2 bytes, 10 in all; five 11-bit codes are 55 bits = 7 bytes: the slot stays packed
    five = np.array([0x4105, 0x4105, 0x3C85, 0x4105, 0x4085] + [0] * 11, dtype=np.uint16)
    buf, _ = C.encode(five)
    assert buf[256] == 1 and list(buf[258:260]) == [7, 0]
    # with eight elements (three more of exponent 130) the byte part needs no padding: 8 + ceil((8 + 4) / 8) = 10
    # bytes against 11 packed: split.  Bytes (d & 1) << 7 | 5; quotients 0, 0, 4, 0, 0, 0, 0, 0 in unary
    eight = np.array([0x4105, 0x4105, 0x3C85, 0x4105, 0x4085, 0x4105, 0x4105, 0x4105] + [0] * 8, dtype=np.uint16)
    buf, defined = C.encode(eight)
    assert buf[256] == 9 and list(buf[258:260]) == [10, 0]
    assert list(buf[272:280]) == [0x05, 0x05, 0x85, 0x05, 0x85, 0x05, 0x05, 0x05]
    assert list(buf[280:282]) == [0xC3, 0x0F]               # bits 1,1,0,0,0,0,1,1 | 1,1,1,1
    assert defined[272:282].all() and not defined[282:SLOT].any()
    assert np.array_equal(C.decode(buf, 16), eight)
    # a byte part that is not a multiple of 4 leaves unspecified padding before the stream
    six = np.array([0x4105] * 6 + [0] * 10, dtype=np.uint16)
    buf, defined = C.encode(six)                            # 6 + 2 padding + 1 = 9 bytes, as many as 66 bits packed: not fewer
    assert buf[256] == 1
    many = np.array([0x4105] * 13 + [0] * 3, dtype=np.uint16)      # 13 + 3 padding + 2 = 18 = ceil(143 / 8): not fewer
    assert C.encode(many)[0][256] == 1
    more = np.array([0x4105] * 14 + [0] * 2, dtype=np.uint16)      # 14 + 2 padding + 2 = 18 < ceil(154 / 8) = 20: split
    buf, defined = C.encode(more)
    assert buf[256] == 9 and list(buf[258:260]) == [18, 0]
    assert defined[272:286].all() and not defined[286:288].any() and defined[288:290].all() and not defined[290:SLOT].any()
    assert list(buf[288:290]) == [0xFF, 0x3F]

    # signed, wide (13 bits): exponents 127, 106, 125 (sign, mantissa 0x11), 128 (mantissa 0x11): span 22;
    # codes sign << 12 | (emax - e) << 7 | mantissa = 0x0080, 0x0B00, 0x1191, 0x0011 at bits 0, 13, 26, 39:
    #   0x80 + (0xB00 << 13) + (0x1191 << 26) + (0x11 << 39) = 0x8C6_4560_0080 -> 52 bits, 7 bytes
    wide = np.array([0, 0x3F80, 0, 0x3500, 0xBE91, 0, 0, 0x4011] + [0] * 8, dtype=np.uint16)
    buf, defined = C.encode(wide)
    assert buf[256] == 1 + 2 + 4 and buf[257] == 128
    assert list(buf[272:279]) == [0x80, 0x00, 0x60, 0x45, 0xC6, 0x08, 0x00]
    assert list(buf[SLOT:SLOT + 4]) == [4, 0xE0, 7, 0]
    assert defined[272:279].all() and not defined[279:SLOT].any()
    assert np.array_equal(C.decode(buf, 16), wide)


def test_mode_follows_the_exponent_span_and_the_signs():
    base = np.zeros(2048, dtype=np.uint16)
    for span, mode in ((0, 1), (15, 1), (16, 3), (31, 3), (32, 0)):
        base[10], base[20] = 0x4000, 0x4000 - (span << 7)   # exponents 128 and 128 - span
        buf, _ = C.encode(base)
        assert buf[256] == mode, span
        assert buf[257] == (128 if mode else 0)
        base[30] = 0x8000 | 0x3F80                          # one negative value: signed, unless raw
        buf, _ = C.encode(base)
        assert buf[256] == (mode | 4 if mode else 0), span
        base[30] = 0
    assert C.encode(np.zeros(2048, dtype=np.uint16))[0][256] == 0      # no non-zero element: raw, nothing to store
    # the mode is per slot
    two = np.zeros(4096, dtype=np.uint16)
    two[5], two[6], two[3000] = 0x3F80, 0x0001, 0x3F80
    buf, _ = C.encode(two)
    assert buf[256] == 0 and buf[SLOT + 256] == 1


def slow_decode(buf, n):
    """Written independently of the oracle's decoder: walks the bitmap bit by bit with a running cursor; packed slots are
    expanded to a string of bits first."""
    out = []
    for s in range((n + 2047) // 2048):
        slot = bytes(buf[s * SLOT:(s + 1) * SLOT])
        mode, emax = slot[256], slot[257]
        ebits, sbit = (5 if mode & 2 else 4), (1 if mode & 4 else 0)
        width = 7 + ebits + sbit
        stream = "".join(format(b, "08b")[::-1] for b in slot[272:]) if mode else ""     # bit k of the stream at index k
        cursor = 0
        if mode & 8:
            # split slot: all quotients at once: the unary stream cut at its one bits gives runs of zeros
            count = sum(bin(b).count("1") for b in slot[:256])
            start = (count + 3) // 4 * 4
            unary = "".join(format(b, "08b")[::-1] for b in slot[272 + start:])
            runs = unary.split("1")[:count]
            assert all(set(r) <= {"0"} for r in runs)
            quot = [len(r) for r in runs]
        for i in range(2048):
            if len(out) == n:
                break
            if slot[i >> 3] & (1 << (i & 7)):
                if mode & 8:
                    b = slot[272 + cursor]
                    out.append((emax - (2 * quot[cursor] + (b >> 7))) * 128 + (b & 127))
                elif mode:
                    field = stream[width * cursor:width * cursor + width]               # low bit first
                    mant = int(field[0:7][::-1], 2)
                    delta = int(field[7:7 + ebits][::-1], 2)
                    sign = int(field[7 + ebits]) if sbit else 0
                    out.append(sign * 32768 + (emax - delta) * 128 + mant)
                else:
                    out.append(slot[272 + 2 * cursor] + 256 * slot[273 + 2 * cursor])
                cursor += 1
            else:
                out.append(0)
    return np.array(out, dtype=np.uint16)


def make_bits(n, density, narrow, seed):
    rng = np.random.default_rng(seed)
    if narrow:      # exponents within 11 (narrow == 1, positive values) or 25 binades (narrow == 2, both signs): every slot packs
        lo = 120 if narrow == 1 else 106
        sign = rng.integers(0, 2, size=n) << 15 if narrow == 2 else 0
        bits = (sign | rng.integers(lo, 131, size=n) << 7 | rng.integers(0, 128, size=n)).astype(np.uint16)
    else:
        bits = rng.integers(1, 65536, size=n, dtype=np.uint32).astype(np.uint16)
    bits[rng.random(n) >= density] = 0
    return bits


@pytest.mark.parametrize("n", [0, 1, 7, 8, 2047, 2048, 2049, 4096, 5000, 9 * 2048])
@pytest.mark.parametrize("density", [0.0, 0.03, 0.5, 1.0])
@pytest.mark.parametrize("narrow", [0, 1, 2])
def test_round_trip_and_invariants(n, density, narrow):
    bits = make_bits(n, density, narrow, 1000 * n + int(100 * density) + narrow)
    if n > 3 and density > 0 and not narrow:
        bits[1], bits[2] = 0x8000, 0x7FC0          # -0.0 and a quiet NaN survive
    buf, defined = C.encode(bits)
    ns = (n + 2047) // 2048
    assert buf.size == C.encoded_bytes(n) == ns * SLOT + (4 * ns + 15) // 16 * 16 + 16
    assert np.array_equal(C.decode(buf, n), bits)
    assert np.array_equal(slow_decode(buf, n), bits)
    moved, ndef = 0, 8
    for s in range(ns):
        chunk = bits[s * 2048:(s + 1) * 2048]
        nz = chunk[chunk != 0]
        nnz = int(nz.size)
        e = (nz >> 7) & 0xFF
        span = int(e.max()) - int(e.min()) if nnz else 0
        mode = 0
        if nnz and span <= 31:
            mode = 1 | (2 if span > 15 else 0) | (4 if (nz >> 15).any() else 0)
        if narrow and nnz:
            assert mode & 1 and (narrow == 2 or mode == 1)
        pad = 0
        if mode:
            width = 7 + (5 if mode & 2 else 4) + (1 if mode & 4 else 0)
            nvb = (width * nnz + 7) // 8
            if not mode & 4:
                # split iff fewer bytes: one per element rounded up to 4, one unary bit per element and per step of 2
                split = (nnz + 3) // 4 * 4 + (nnz + int(((int(e.max()) - e.astype(np.int64)) >> 1).sum()) + 7) // 8
                if split < nvb:
                    mode, nvb, pad = 9, split, (nnz + 3) // 4 * 4 - nnz
        cnt = buf[ns * SLOT + 4 * s:ns * SLOT + 4 * s + 4]
        assert int(cnt[0]) + 256 * int(cnt[1]) == nnz + (0x8000 if mode & 1 else 0) + (0x4000 if mode & 2 else 0) + (0x2000 if mode & 4 else 0) + (0x1000 if mode & 8 else 0)
        assert int(np.unpackbits(buf[s * SLOT:s * SLOT + 256]).sum()) == nnz
        assert buf[s * SLOT + 256] == mode
        if mode:
            assert buf[s * SLOT + 257] == int(e.max())
        else:
            vals = buf[s * SLOT + 272:s * SLOT + 272 + 2 * nnz].view(np.uint16)
            assert np.array_equal(vals, nz)                     # order kept, no zero stored
            nvb = 2 * nnz
        assert int(cnt[2]) + 256 * int(cnt[3]) == nvb == int(buf[s * SLOT + 258]) + 256 * int(buf[s * SLOT + 259])
        moved += 272 + (nvb + 15) // 16 * 16
        ndef += 256 + 4 + nvb - pad + 4
    assert C.moved_bytes(buf, n) == moved
    t = C.trailer_offset(n)
    assert t == ns * SLOT + (4 * ns + 15) // 16 * 16
    assert sum(int(b) << (8 * i) for i, b in enumerate(buf[t:t + 8])) == moved
    assert int(defined.sum()) == ndef


def test_garbage_in_unspecified_bytes_is_ignored():
    for narrow in (0, 1, 2):
        bits = make_bits(3000, 0.6, narrow, 7)
        buf, defined = C.encode(bits)
        buf = buf.copy()
        buf[~defined] = 0xAB
        assert np.array_equal(C.decode(buf, 3000), bits)


def test_relu_output_traffic():
    # a ReLU output of a symmetric distribution is half zeros and has no sign bits: 1/16 bitmap + header + 1/2 of the
    # values; packed they would take 11 bits (12 where a slot of about 1024 half-normal values has one more than 15
    # binades below the largest: about one slot in four), split they take 8 bits and a unary quotient of 1.8 bits on
    # average (half-normal magnitudes: P(d >> 1 = 0, 1, 2, ...) = 0.4, 0.43, 0.12, ...): 0.37 to 0.39 of the plain bytes.
    import workloads as W
    x = W.rng.normal(99, (64 * 2048,))
    bits = W.rng.bf16_bits(np.maximum(x, 0.0))
    buf, _ = C.encode(bits)
    ratio = C.moved_bytes(buf, bits.size) / (2.0 * bits.size)
    modes = [int(buf[s * SLOT + 256]) for s in range(64)]
    assert all(m == 9 for m in modes)
    assert 0.37 < ratio < 0.39
