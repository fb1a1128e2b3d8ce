"""Pins of the swap-encoding oracle: a hand-written example, the inverse property on edge cases, an independent
bit-by-bit decoder, and structural invariants of the format."""
import numpy as np
import pytest

from oracle import swap_codec as C


def test_hand_written_example():
    # 16 elements: non-zeros at 1, 3, 4, 7 and 15 (-0.0 = 0x8000 and a NaN pattern count as non-zero)
    bits = np.array([0, 0x3F80, 0, 0x8000, 0x7FC1, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0, 0xFFFF], dtype=np.uint16)
    buf, defined = C.encode(bits)
    assert buf.size == 4368 + 16
    assert list(buf[4368:4376]) == [0x20, 0x01, 0, 0, 0, 0, 0, 0]    # 288 = 16 + 256 + 16, little-endian
    assert defined[4368:4376].all() and not defined[4376:].any()
    assert list(buf[:4]) == [5, 0, 0, 0]
    assert buf[16] == 0b10011010 and buf[17] == 0b10000000 and not buf[18:272].any()
    assert list(buf[272:282]) == [0x80, 0x3F, 0x00, 0x80, 0xC1, 0x7F, 0x01, 0x00, 0xFF, 0xFF]
    assert defined[:4].all() and not defined[4:16].any() and defined[16:282].all() and not defined[282:4368].any()
    assert np.array_equal(C.decode(buf, 16), bits)
    assert C.moved_bytes(buf, 16) == 16 + 256 + 16


def slow_decode(buf, n):
    """Written independently of the oracle's decoder: walks the bitmap bit by bit with a running value cursor."""
    out = []
    for s in range((n + 2047) // 2048):
        slot = bytes(buf[s * 4368:(s + 1) * 4368])
        cursor = 272
        for i in range(2048):
            if len(out) == n:
                break
            if slot[16 + (i >> 3)] & (1 << (i & 7)):
                out.append(slot[cursor] + 256 * slot[cursor + 1])
                cursor += 2
            else:
                out.append(0)
    return np.array(out, dtype=np.uint16)


@pytest.mark.parametrize("n", [0, 1, 7, 8, 2047, 2048, 2049, 4096, 5000])
@pytest.mark.parametrize("density", [0.0, 0.03, 0.5, 1.0])
def test_round_trip_and_invariants(n, density):
    rng = np.random.default_rng(1000 * n + int(100 * density))
    bits = rng.integers(1, 65536, size=n, dtype=np.uint32).astype(np.uint16)
    bits[rng.random(n) >= density] = 0
    if n > 3 and density > 0:
        bits[1], bits[2] = 0x8000, 0x7FC0          # -0.0 and a quiet NaN survive
    buf, defined = C.encode(bits)
    assert buf.size == C.encoded_bytes(n) == (n + 2047) // 2048 * 4368 + 16
    assert np.array_equal(C.decode(buf, n), bits)
    assert np.array_equal(slow_decode(buf, n), bits)
    moved = 0
    for s in range(C.slots(n)):
        chunk = bits[s * 2048:(s + 1) * 2048]
        nnz = int(np.count_nonzero(chunk))
        head = buf[s * 4368:s * 4368 + 4]
        assert int(head[0]) + 256 * int(head[1]) + 65536 * int(head[2]) == nnz
        bitmap = buf[s * 4368 + 16:s * 4368 + 272]
        assert int(np.unpackbits(bitmap).sum()) == nnz
        vals = buf[s * 4368 + 272:s * 4368 + 272 + 2 * nnz].view(np.uint16)
        assert np.array_equal(vals, chunk[chunk != 0])          # order kept, no zero stored
        moved += 272 + (2 * nnz + 15) // 16 * 16
    assert C.moved_bytes(buf, n) == moved
    trailer = buf[C.slots(n) * 4368:C.slots(n) * 4368 + 8]
    assert sum(int(b) << (8 * i) for i, b in enumerate(trailer)) == moved
    assert int(defined.sum()) == 8 + sum(4 + 256 + 2 * int(np.count_nonzero(bits[s * 2048:(s + 1) * 2048])) for s in range(C.slots(n)))


def test_garbage_after_the_values_is_ignored():
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 3, size=3000, dtype=np.uint32).astype(np.uint16)
    buf, defined = C.encode(bits)
    buf = buf.copy()
    buf[~defined] = 0xAB
    assert np.array_equal(C.decode(buf, 3000), bits)


def test_relu_output_halves_the_traffic():
    # a ReLU output of a symmetric distribution is half zeros: 1/16 bitmap + 1/2 values of the plain size
    import workloads as W
    x = W.rng.normal(99, (64 * 2048,))
    bits = W.rng.bf16_bits(np.maximum(x, 0.0))
    buf, _ = C.encode(bits)
    ratio = C.moved_bytes(buf, bits.size) / (2.0 * bits.size)
    assert 0.54 < ratio < 0.59
