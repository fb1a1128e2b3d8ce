"""Swap encoding on the GPU against the oracle's encoding: the bytes the format defines must be identical, decoding
the oracle's bytes must return the tensor, and a swapping run that encodes must stay bit-identical."""
import numpy as np
import pytest

import workloads as W
from oracle import swap_codec as C

pytestmark = pytest.mark.gpu


def tensors_for(case, n):
    rng = np.random.default_rng(n + 17)
    if case == "relu":
        return W.rng.bf16_bits(np.maximum(W.rng.normal(1234 + n, (n,)), 0.0))
    if case == "zeros":
        return np.zeros(n, dtype=np.uint16)
    if case == "dense":
        return rng.integers(1, 65536, size=n, dtype=np.uint32).astype(np.uint16)
    if case == "narrow":       # no zeros, exponents within 11 binades, both signs: every slot is packed
        return (rng.integers(0, 2, size=n) << 15 | rng.integers(120, 131, size=n) << 7 | rng.integers(0, 128, size=n)).astype(np.uint16)
    if case == "wide":         # 70 % non-zero, exponents within 26 binades, both signs: 13-bit codes
        bits = (rng.integers(0, 2, size=n) << 15 | rng.integers(100, 126, size=n) << 7 | rng.integers(0, 128, size=n)).astype(np.uint16)
        bits[rng.random(n) < 0.3] = 0
        return bits
    if case == "span":         # 30 % non-zero, positive; slots alternate between an exponent span of 15 (4-bit differences) and 16 (5-bit)
        e = rng.integers(100, 116, size=n)
        e[1000::4096], e[1001::4096] = 100, 115
        e[3000::4096], e[3001::4096] = 99, 115
        bits = (e << 7 | rng.integers(0, 128, size=n)).astype(np.uint16)
        keep = rng.random(n) < 0.3
        keep[1000::4096] = keep[1001::4096] = keep[3000::4096] = keep[3001::4096] = True
        bits[~keep] = 0
        return bits
    bits = rng.integers(0, 65536, size=n, dtype=np.uint32).astype(np.uint16)      # "mixed": 90 % zeros, -0.0, NaNs
    bits[rng.random(n) < 0.9] = 0
    bits[::97] = 0x8000
    bits[5::101] = 0x7FC0
    return bits


@pytest.mark.parametrize("n", [8, 2040, 2048, 2056, 8 * 2048, 300000, 1234568])
@pytest.mark.parametrize("case", ["relu", "zeros", "dense", "mixed", "narrow", "wide", "span"])
def test_encode_and_decode_match_the_oracle(case, n):
    import torch
    import paper_1807_02037_amd as L
    bits = tensors_for(case, n)
    ref, defined = C.encode(bits)
    nbytes = L.swap_encoded_bytes(n)
    assert nbytes == ref.size == C.encoded_bytes(n)
    src = torch.from_numpy(bits.view(np.int16).copy()).cuda()
    host = torch.full((nbytes,), 0x5A, dtype=torch.uint8).pin_memory()
    stream = torch.cuda.current_stream().cuda_stream
    L.swap_encode(host.data_ptr(), src.data_ptr(), n, stream)
    torch.cuda.synchronize()
    got = host.numpy()
    assert np.array_equal(got[defined], ref[defined])
    assert L.swap_moved_bytes(host.data_ptr(), n) == C.moved_bytes(ref, n)      # trailer (also among the defined bytes)
    # decode what the GPU wrote
    dst = torch.full((n,), -1, dtype=torch.int16, device="cuda")
    L.swap_decode(dst.data_ptr(), host.data_ptr(), n, stream)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy().view(np.uint16), bits)
    # decode what the oracle wrote, with the unspecified bytes filled with a pattern
    filled = ref.copy()
    filled[~defined] = 0xC3
    host2 = torch.from_numpy(filled).pin_memory()
    dst.fill_(-1)
    L.swap_decode(dst.data_ptr(), host2.data_ptr(), n, stream)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy().view(np.uint16), bits)


def draw_bits(rng, kind, n):
    if kind == 0:        # arbitrary bit patterns
        bits = rng.integers(0, 65536, size=n, dtype=np.uint32).astype(np.uint16)
    elif kind == 1:      # both signs, a random exponent window of 1 to 40 binades
        lo, span = int(rng.integers(0, 230)), int(rng.integers(1, 40))
        bits = (rng.integers(0, 2, size=n) << 15 | rng.integers(lo, min(lo + span, 256), size=n) << 7 | rng.integers(0, 128, size=n)).astype(np.uint16)
    elif kind == 2:      # ReLU outputs at a random scale
        x = np.maximum(rng.normal(size=n) * 10.0 ** rng.uniform(-3, 3), 0)
        bits = (x.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    else:                # heavy-tailed values of both signs
        x = rng.normal(size=n) * np.exp(rng.normal(size=n) * 3)
        bits = (x.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    bits[rng.random(n) < rng.uniform(0, 0.95)] = 0
    return bits


@pytest.mark.parametrize("it", range(24))
def test_random_tensors_match_the_oracle_and_round_trip(it):
    import torch
    import paper_1807_02037_amd as L
    rng = np.random.default_rng(4200 + it)
    n = 8 * int(rng.integers(1, 4000))
    bits = draw_bits(rng, it % 4, n)
    ref, defined = C.encode(bits)
    src = torch.from_numpy(bits.view(np.int16).copy()).cuda()
    host = torch.full((L.swap_encoded_bytes(n),), 0x5A, dtype=torch.uint8).pin_memory()
    stream = torch.cuda.current_stream().cuda_stream
    L.swap_encode(host.data_ptr(), src.data_ptr(), n, stream)
    dst = torch.full((n,), -1, dtype=torch.int16, device="cuda")
    L.swap_decode(dst.data_ptr(), host.data_ptr(), n, stream)
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy()[defined], ref[defined])
    assert L.swap_moved_bytes(host.data_ptr(), n) == C.moved_bytes(ref, n)
    assert np.array_equal(dst.cpu().numpy().view(np.uint16), bits)


def test_bad_arguments_are_errors():
    import torch
    import paper_1807_02037_amd as L
    t = torch.zeros(64, dtype=torch.int16, device="cuda")
    h = torch.zeros(8192, dtype=torch.uint8).pin_memory()
    with pytest.raises(L.LmsError):
        L.swap_encode(h.data_ptr(), t.data_ptr(), 12, 0)          # not a multiple of 8
    with pytest.raises(L.LmsError):
        L.swap_decode(t.data_ptr() + 2, h.data_ptr(), 8, 0)        # misaligned


def test_encoded_swapping_moves_fewer_bytes_and_stays_bit_identical():
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    spec = W.bottleneck_stage(batch=4)
    tensors = W.make_tensors(spec)
    base = Session(spec, tensors)
    loss0, _ = base.step()
    g0 = base.grad_bits()
    rw = dict(budget_bytes=int(base.unswapped_need * 0.75), fuse_swapins=1, ctrld_strategy=A.OWN)
    del base
    plain = Session(spec, tensors, rewrite=rw)
    _, st_plain = plain.step()
    del plain
    enc = Session(spec, tensors, rewrite=rw, flags=A.X_ENCODE_SWAPS)
    for _ in range(2):
        loss1, st = enc.step()
    assert np.float32(loss1).view(np.uint32) == np.float32(loss0).view(np.uint32)
    g1 = enc.grad_bits()
    for k in g0:
        assert np.array_equal(g0[k], g1[k]), k
    assert st.bytes_d2h == st.bytes_h2d > 0
    # ReLU outputs of the randomly initialised stage are about half zeros: bitmap (1/16) + values (about 1/2), the
    # values of packed slots at 3/4 of their size
    assert 0.38 * st_plain.bytes_d2h < st.bytes_d2h < 0.62 * st_plain.bytes_d2h
