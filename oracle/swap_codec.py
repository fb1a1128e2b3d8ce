"""Oracle for the lossless swap encoding: test infrastructure only (fp64 / integer reference on the CPU;
only tests, the smoke check and the benchmark's CPU leg may import this package).

Section 4.2.1 (Eq. 3-5) of the paper writes the swap as id = f^-1 o f and remarks that an encoding /
decoding pair may take the place of the two identities.  The pair here exploits that tensors which cross
from the forward to the backward phase are outputs of ReLU and hold many exact zeros: a tensor of 16-bit
elements is cut into slots of 2048 elements; a slot is stored as

    bytes [0, 256)    bitmap: bit (i % 8) of byte i // 8 is set iff element i of the slot is not 0x0000
    bytes [256, ...)  the non-zero elements in order, little-endian u16

and slot s starts at byte s * 4352 (= 256 + 2 * 2048, the size of a slot without any zero), so slots can be
written and read independently.  After the last slot come
    counts   one little-endian u16 per slot: its number of non-zero elements (0..2048),
             the region padded to a multiple of 16 bytes;
    trailer  16 bytes: the number of slot bytes a copy has to move (per slot the bitmap and the values rounded
             up to 16 bytes) as little-endian u64, then 8 unused bytes.
"Zero" is the bit pattern 0x0000 only: -0.0 (0x8000), NaNs and denormals are kept as they are, so
decode(encode(t)) == t bit for bit.  Elements past the end of the tensor in the last slot count as zeros.
Bytes of a slot after its last value, and padding, are unspecified.
"""
import numpy as np

SLOT_ELEMENTS = 2048
BITMAP_BYTES = SLOT_ELEMENTS // 8
SLOT_BYTES = BITMAP_BYTES + 2 * SLOT_ELEMENTS
TRAILER_BYTES = 16


def slots(n):
    return (n + SLOT_ELEMENTS - 1) // SLOT_ELEMENTS


def counts_offset(n):
    return slots(n) * SLOT_BYTES


def trailer_offset(n):
    return counts_offset(n) + (2 * slots(n) + 15) // 16 * 16


def encoded_bytes(n):
    """Size of the host buffer an n-element tensor needs (every slot at its largest, counts, trailer)."""
    return trailer_offset(n) + TRAILER_BYTES


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
        for j, v in enumerate(nz):
            out[base + BITMAP_BYTES + 2 * j] = v & 0xFF
            out[base + BITMAP_BYTES + 2 * j + 1] = v >> 8
        defined[base:base + BITMAP_BYTES + 2 * len(nz)] = True
        c = counts_offset(n) + 2 * s
        out[c], out[c + 1] = len(nz) & 0xFF, len(nz) >> 8
        defined[c:c + 2] = True
        moved += BITMAP_BYTES + (2 * len(nz) + 15) // 16 * 16
    t = trailer_offset(n)
    out[t:t + 8] = np.frombuffer(np.uint64(moved).tobytes(), dtype=np.uint8)
    defined[t:t + 8] = True
    return out, defined


def decode(buf, n):
    """Inverse of encode: uint8 array, element count -> uint16 array of n elements (reads bitmaps and values only)."""
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    out = np.zeros(n, dtype=np.uint16)
    for s in range(slots(n)):
        base = s * SLOT_BYTES
        j = 0
        for i in range(min(SLOT_ELEMENTS, n - s * SLOT_ELEMENTS)):
            if buf[base + i // 8] >> (i % 8) & 1:
                p = base + BITMAP_BYTES + 2 * j
                out[s * SLOT_ELEMENTS + i] = int(buf[p]) | (int(buf[p + 1]) << 8)
                j += 1
    return out


def moved_bytes(buf, n):
    """Slot bytes of the encoded buffer that a copy has to move, recomputed from the bitmaps."""
    total = 0
    for s in range(slots(n)):
        nnz = int(np.unpackbits(buf[s * SLOT_BYTES:s * SLOT_BYTES + BITMAP_BYTES]).sum())
        total += BITMAP_BYTES + (2 * nnz + 15) // 16 * 16
    return total
