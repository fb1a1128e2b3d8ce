"""Pins of the swap-encoding oracle: a hand-written example, the inverse property on edge cases, an independent
bit-by-bit decoder, and structural invariants of the format."""
import numpy as np
import pytest

from oracle import swap_codec as C


def test_hand_written_example():
    # 16 elements: non-zeros at 1, 3, 4, 7 and 15 (-0.0 = 0x8000 and a NaN pattern count as non-zero)
    bits = np.array([0, 0x3F80, 0, 0x8000, 0x7FC1, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0, 0xFFFF], dtype=np.uint16)
    buf, defined = C.encode(bits)
    assert buf.size == 4352 + 16 + 16                       # one slot, counts padded to 16, trailer
    assert buf[0] == 0b10011010 and buf[1] == 0b10000000 and not buf[2:256].any()
    assert list(buf[256:266]) == [0x80, 0x3F, 0x00, 0x80, 0xC1, 0x7F, 0x01, 0x00, 0xFF, 0xFF]
    assert list(buf[4352:4354]) == [5, 0]                   # count of the only slot
    assert list(buf[4368:4376]) == [0x10, 0x01, 0, 0, 0, 0, 0, 0]    # 272 = 256 + 16, little-endian
    assert defined[:266].all() and not defined[266:4352].any() and defined[4352:4354].all() and not defined[4354:4368].any()
    assert defined[4368:4376].all() and not defined[4376:].any()
    assert np.array_equal(C.decode(buf, 16), bits)
    assert C.moved_bytes(buf, 16) == 256 + 16


def slow_decode(buf, n):
    """Written independently of the oracle's decoder: walks the bitmap bit by bit with a running value cursor."""
    out = []
    for s in range((n + 2047) // 2048):
        slot = bytes(buf[s * 4352:(s + 1) * 4352])
        cursor = 256
        for i in range(2048):
            if len(out) == n:
                break
            if slot[i >> 3] & (1 << (i & 7)):
                out.append(slot[cursor] + 256 * slot[cursor + 1])
                cursor += 2
            else:
                out.append(0)
    return np.array(out, dtype=np.uint16)


@pytest.mark.parametrize("n", [0, 1, 7, 8, 2047, 2048, 2049, 4096, 5000, 9 * 2048])
@pytest.mark.parametrize("density", [0.0, 0.03, 0.5, 1.0])
def test_round_trip_and_invariants(n, density):
    rng = np.random.default_rng(1000 * n + int(100 * density))
    bits = rng.integers(1, 65536, size=n, dtype=np.uint32).astype(np.uint16)
    bits[rng.random(n) >= density] = 0
    if n > 3 and density > 0:
        bits[1], bits[2] = 0x8000, 0x7FC0          # -0.0 and a quiet NaN survive
    buf, defined = C.encode(bits)
    ns = (n + 2047) // 2048
    assert buf.size == C.encoded_bytes(n) == ns * 4352 + (2 * ns + 15) // 16 * 16 + 16
    assert np.array_equal(C.decode(buf, n), bits)
    assert np.array_equal(slow_decode(buf, n), bits)
    moved = 0
    for s in range(ns):
        chunk = bits[s * 2048:(s + 1) * 2048]
        nnz = int(np.count_nonzero(chunk))
        cnt = buf[ns * 4352 + 2 * s:ns * 4352 + 2 * s + 2]
        assert int(cnt[0]) + 256 * int(cnt[1]) == nnz
        assert int(np.unpackbits(buf[s * 4352:s * 4352 + 256]).sum()) == nnz
        vals = buf[s * 4352 + 256:s * 4352 + 256 + 2 * nnz].view(np.uint16)
        assert np.array_equal(vals, chunk[chunk != 0])          # order kept, no zero stored
        moved += 256 + (2 * nnz + 15) // 16 * 16
    assert C.moved_bytes(buf, n) == moved
    t = C.trailer_offset(n)
    assert t == ns * 4352 + (2 * ns + 15) // 16 * 16
    assert sum(int(b) << (8 * i) for i, b in enumerate(buf[t:t + 8])) == moved
    assert int(defined.sum()) == 8 + sum(256 + 2 + 2 * int(np.count_nonzero(bits[s * 2048:(s + 1) * 2048])) for s in range(ns))


def test_garbage_in_unspecified_bytes_is_ignored():
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
