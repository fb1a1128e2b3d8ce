"""Oracle for the lossless swap encoding: test infrastructure only (fp64 / integer reference on the CPU;
only tests, the smoke check and the benchmark's CPU leg may import this package).

Section 4.2.1 (Eq. 3-5) of the paper writes the swap as id = f^-1 o f and remarks that an encoding /
decoding pair may take the place of the two identities.  The pair here exploits two properties of the tensors
that cross from the forward to the backward phase: they are outputs of ReLU and hold many exact zeros, and the
exponents of the values of one neighbourhood span few binades.  A tensor of 16-bit elements (bfloat16 bit
patterns: sign, 8 exponent bits, 7 mantissa bits) is cut into slots of 2048 elements; a slot is stored as

    bytes [0, 256)    bitmap: bit (i % 8) of byte i // 8 is set iff element i of the slot is not 0x0000
    byte  256         mode: 0 = raw values; else bit 0 set = packed values, bit 1 = wide exponent difference (5 bits
                      instead of 4), bit 2 = signed (a sign bit per value), bit 3 = split (see below)
    byte  257         emax: the largest exponent field among the non-zero elements (packed; 0 in raw mode)
    bytes [258, 260)  little-endian u16: the number of value bytes of the slot
    bytes [260, 272)  unspecified
    bytes [272, ...)  the non-zero elements in order:
                      raw     little-endian u16 each
                      packed  codes of B = 7 + (5 if wide else 4) + (1 if signed else 0) bits (11 to 13):
                              sign << (B - 1) | (emax - exponent) << 7 | mantissa, the sign only if signed, as a
                              little-endian bit stream: code j occupies bits [B j, B j + B) of the stream, byte b
                              holds the stream bits [8 b, 8 b + 8); unused bits of the last byte are zero
                      split   with d = emax - exponent (0..31): one byte per element, (d & 1) << 7 | mantissa;
                              unspecified bytes up to the next multiple of 4; then the quotients d >> 1 in unary, as
                              a little-endian bit stream like the one above: element j adds (d >> 1) zero bits and
                              a one bit; unused bits of the last byte are zero

A slot is packed iff it has a non-zero element and the exponent fields of all its non-zero elements lie within
31 of the largest one; it is wide iff they do not all lie within 15, and signed iff a non-zero element has its
sign bit set (the outputs of ReLU never have).  The code then holds every bit of the element: the pair stays
lossless for any bit pattern, NaNs, infinities and denormals included.  Any other slot is raw.  A packed slot
without signs is stored split (mode = packed | split, the wide bit clear) iff that takes fewer value bytes: the
magnitudes of one neighbourhood crowd just below the largest, so small differences are frequent and the unary
quotient with one remainder bit (a Rice code) takes about 2.8 bits per element where the fixed field takes 4 or 5.  Slot s starts at
byte s * 4368 (= 256 + 16 + 2 * 2048, the size of a raw slot without any zero), so slots can be written and read
independently.  After the last slot come
    counts   one little-endian u32 per slot: its number of non-zero elements (0..2048) in bits 0-11, bit 15 set for
             a packed slot, bit 14 for wide, bit 13 for signed, bit 12 for split, its number of value bytes in bits
             16-31; the region padded to a multiple of 16 bytes;
    trailer  16 bytes: the number of slot bytes a copy has to move (per slot bitmap, header and the value bytes
             rounded up to 16 bytes) as little-endian u64, then 8 unused bytes.
"Zero" is the bit pattern 0x0000 only: -0.0 (0x8000), NaNs and denormals are kept as they are, so
decode(encode(t)) == t bit for bit.  Elements past the end of the tensor in the last slot count as zeros.
Bytes of a slot after its last value byte, and padding, are unspecified.
"""
import numpy as np

SLOT_ELEMENTS = 2048
BITMAP_BYTES = SLOT_ELEMENTS // 8
HEADER_BYTES = 16
VALUES_AT = BITMAP_BYTES + HEADER_BYTES
SLOT_BYTES = VALUES_AT + 2 * SLOT_ELEMENTS
TRAILER_BYTES = 16
NARROW_SPAN, WIDE_SPAN = 15, 31      # exponent spans that 4 and 5 bits of difference cover
PACKED, WIDE, SIGNED, SPLIT = 1, 2, 4, 8       # bits of the mode byte


def slots(n):
    return (n + SLOT_ELEMENTS - 1) // SLOT_ELEMENTS


def counts_offset(n):
    return slots(n) * SLOT_BYTES


def trailer_offset(n):
    return counts_offset(n) + (4 * slots(n) + 15) // 16 * 16


def encoded_bytes(n):
    """Size of the host buffer an n-element tensor needs (every slot at its largest, counts, trailer)."""
    return trailer_offset(n) + TRAILER_BYTES


def code_bits(mode):
    return 7 + (5 if mode & WIDE else 4) + (1 if mode & SIGNED else 0)


def value_bytes(nnz, mode, quotients=0):
    """quotients: sum of d >> 1 over the slot's elements (split slots only)."""
    if mode & SPLIT:
        return (nnz + 3) // 4 * 4 + (nnz + quotients + 7) // 8
    return (code_bits(mode) * nnz + 7) // 8 if mode & PACKED else 2 * nnz


def count_word(nnz, mode, nbytes):
    return (nnz | (0x8000 if mode & PACKED else 0) | (0x4000 if mode & WIDE else 0) | (0x2000 if mode & SIGNED else 0)
            | (0x1000 if mode & SPLIT else 0) | nbytes << 16)


def exponent(v):
    return (v >> 7) & 0xFF


def encode(bits):
    """bits: uint16 array -> (uint8 array of encoded_bytes(n), defined: bool array marking specified bytes)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16).ravel()
    n = bits.size
    out = np.zeros(encoded_bytes(n), dtype=np.uint8)
    defined = np.zeros(out.size, dtype=bool)
    moved = 0
    for s in range(slots(n)):
        chunk = bits[s * SLOT_ELEMENTS:(s + 1) * SLOT_ELEMENTS]
        base = s * SLOT_BYTES
        nz = [int(v) for v in chunk if v != 0]
        for i, v in enumerate(chunk):
            if v != 0:
                out[base + i // 8] |= np.uint8(1 << (i % 8))
        emax = max((exponent(v) for v in nz), default=0)
        emin = min((exponent(v) for v in nz), default=0)
        mode = 0
        quotients = 0
        if nz and emax - emin <= WIDE_SPAN:
            mode = PACKED | (WIDE if emax - emin > NARROW_SPAN else 0) | (SIGNED if any(v >> 15 for v in nz) else 0)
            quotients = sum((emax - exponent(v)) >> 1 for v in nz)
            if not mode & SIGNED and value_bytes(len(nz), PACKED | SPLIT, quotients) < value_bytes(len(nz), mode):
                mode = PACKED | SPLIT
        out[base + BITMAP_BYTES] = mode
        out[base + BITMAP_BYTES + 1] = emax if mode else 0
        nvb = value_bytes(len(nz), mode, quotients)
        out[base + BITMAP_BYTES + 2] = nvb & 0xFF
        out[base + BITMAP_BYTES + 3] = nvb >> 8
        if mode & SPLIT:
            first = (len(nz) + 3) // 4 * 4             # where the unary stream starts
            stream, at = 0, 0
            for j, v in enumerate(nz):
                d = emax - exponent(v)
                out[base + VALUES_AT + j] = (d & 1) << 7 | (v & 0x7F)
                at += d >> 1
                stream |= 1 << at
                at += 1
            for b in range((at + 7) // 8):
                out[base + VALUES_AT + first + b] = (stream >> (8 * b)) & 0xFF
        elif mode:
            nbits = code_bits(mode)
            stream = 0                                   # the bit stream as one integer, bit 0 first
            for j, v in enumerate(nz):
                code = (emax - exponent(v)) << 7 | (v & 0x7F)
                if mode & SIGNED:
                    code |= (v >> 15) << (nbits - 1)
                stream |= code << (nbits * j)
            for b in range(value_bytes(len(nz), mode)):
                out[base + VALUES_AT + b] = (stream >> (8 * b)) & 0xFF
        else:
            for j, v in enumerate(nz):
                out[base + VALUES_AT + 2 * j] = v & 0xFF
                out[base + VALUES_AT + 2 * j + 1] = v >> 8
        defined[base:base + BITMAP_BYTES + 4] = True
        defined[base + VALUES_AT:base + VALUES_AT + nvb] = True
        if mode & SPLIT:
            defined[base + VALUES_AT + len(nz):base + VALUES_AT + (len(nz) + 3) // 4 * 4] = False
        c = counts_offset(n) + 4 * s
        word = count_word(len(nz), mode, nvb)
        out[c:c + 4] = [(word >> (8 * b)) & 0xFF for b in range(4)]
        defined[c:c + 4] = True
        moved += VALUES_AT + (nvb + 15) // 16 * 16
    t = trailer_offset(n)
    out[t:t + 8] = np.frombuffer(np.uint64(moved).tobytes(), dtype=np.uint8)
    defined[t:t + 8] = True
    return out, defined


def decode(buf, n):
    """Inverse of encode: uint8 array, element count -> uint16 array of n elements (reads bitmaps, headers and
    values only)."""
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    out = np.zeros(n, dtype=np.uint16)
    for s in range(slots(n)):
        base = s * SLOT_BYTES
        mode = int(buf[base + BITMAP_BYTES])
        emax = int(buf[base + BITMAP_BYTES + 1])
        nbits = code_bits(mode)
        j = 0
        nnz = int(sum(bin(int(b)).count("1") for b in buf[base:base + BITMAP_BYTES]))
        first = base + VALUES_AT + (nnz + 3) // 4 * 4          # split slots: the unary stream and a cursor into it
        ubit = 0
        for i in range(min(SLOT_ELEMENTS, n - s * SLOT_ELEMENTS)):
            if buf[base + i // 8] >> (i % 8) & 1:
                if mode & SPLIT:
                    q = 0
                    while not (int(buf[first + ubit // 8]) >> (ubit % 8)) & 1:
                        q += 1
                        ubit += 1
                    ubit += 1
                    byte = int(buf[base + VALUES_AT + j])
                    v = (emax - (2 * q + (byte >> 7))) << 7 | (byte & 0x7F)
                elif mode & PACKED:
                    bit = nbits * j
                    p = base + VALUES_AT + bit // 8
                    word = int(buf[p]) | (int(buf[p + 1]) << 8) | (int(buf[p + 2]) << 16 if bit % 8 + nbits > 16 else 0)
                    code = (word >> (bit % 8)) & ((1 << nbits) - 1)
                    delta = (code >> 7) & (31 if mode & WIDE else 15)
                    sign = code >> (nbits - 1) if mode & SIGNED else 0
                    v = sign << 15 | (emax - delta) << 7 | (code & 0x7F)
                else:
                    p = base + VALUES_AT + 2 * j
                    v = int(buf[p]) | (int(buf[p + 1]) << 8)
                out[s * SLOT_ELEMENTS + i] = v
                j += 1
    return out


def moved_bytes(buf, n):
    """Slot bytes of the encoded buffer that a copy has to move, from the value-byte counts in the slot headers."""
    total = 0
    for s in range(slots(n)):
        base = s * SLOT_BYTES
        nvb = int(buf[base + BITMAP_BYTES + 2]) | int(buf[base + BITMAP_BYTES + 3]) << 8
        total += VALUES_AT + (nvb + 15) // 16 * 16
    return total
