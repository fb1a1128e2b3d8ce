"""Encoded swaps that cross the host link through the copy engines (LMS_X_STAGED_SWAPS): swap operations stay
identities (Eq. 2 / Eq. 5), so a run must equal the unswapped run bit for bit whatever staged width the executor
picked, also when the data changes between steps and slots outgrow the width chosen from the previous step."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def same_bits(a, b):
    return np.float32(a).view(np.uint32) == np.float32(b).view(np.uint32)


NETS = [("cfg2_stage_small", lambda: W.bottleneck_stage(batch=4, size=28, width=64)),
        ("resnet_small", lambda: W.resnet50(batch=4, size=64)),
        ("unet_small", lambda: W.unet3d(batch=1, size=32))]


@pytest.mark.parametrize("name,make", NETS, ids=[n for n, _ in NETS])
def test_staged_swaps_are_bit_identical_over_steps_with_changing_data(name, make):
    import torch
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    spec = make()
    tensors = W.make_tensors(spec, affine="random") if spec["cfg"] == 3 else W.make_tensors(spec)
    base = Session(spec, tensors)
    sw = Session(spec, tensors, rewrite=dict(n_tensors=-1, fuse_swapins=1), flags=A.X_ENCODE_SWAPS | A.X_STAGED_SWAPS)
    assert sw.rewrite_stats.tensors_swapped > 0
    assert sw.arena_bytes >= L.swap_staging_bytes()
    x_name = spec["input"][0]
    moved = []
    # steps 0, 1: the same batch (step 0 moves directly, step 1 with the width step 0 gave); step 2: the negated
    # batch, step 3: a much sparser one (widths from the step before no longer fit / are too wide), step 4 again
    for step in range(5):
        if step in (2, 3):
            for s in (base, sw):
                x = s.dev[x_name]
                if step == 2:
                    x.neg_()
                else:
                    x.mul_((torch.arange(x.numel(), device="cuda").reshape(x.shape) % 7 == 0).to(x.dtype))
        lb, _ = base.step()
        ls, st = sw.step()
        assert np.isfinite(lb) and same_bits(lb, ls), step
        gb, gs = base.grad_bits(), sw.grad_bits()
        assert len(gb) == len(gs) > 0
        for k in gb:
            assert np.array_equal(gb[k], gs[k]), (step, k)
        assert st.bytes_d2h == st.bytes_h2d > 0
        moved.append(st.bytes_d2h)
    # a staged transfer moves whole widths: never less than the direct one of the same data, and not much more
    assert moved[0] <= moved[1] <= 1.25 * moved[0]


def test_staged_swaps_need_their_share_of_the_arena():
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    spec = W.bottleneck_stage(batch=2, size=16, width=32)
    tensors = W.make_tensors(spec)
    plain = Session(spec, tensors, rewrite=dict(n_tensors=-1, fuse_swapins=1), flags=A.X_ENCODE_SWAPS)
    with pytest.raises(L.LmsError):
        Session(spec, tensors, rewrite=dict(n_tensors=-1, fuse_swapins=1), flags=A.X_ENCODE_SWAPS | A.X_STAGED_SWAPS,
                arena_bytes=plain.arena_bytes)


def test_swap_grid_changes_no_bit_and_is_range_checked():
    """lms_exec_set_swap_grid: the work-groups of the encoding / decoding kernels are a launch shape, not part of the
    encoding: every setting gives the unswapped run's loss and gradients; values outside 0..4096 are refused."""
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    spec = W.bottleneck_stage(batch=4, size=28, width=64)
    tensors = W.make_tensors(spec)
    base = Session(spec, tensors)
    lb, _ = base.step()
    gb = base.grad_bits()
    sw = Session(spec, tensors, rewrite=dict(n_tensors=-1, fuse_swapins=1), flags=A.X_ENCODE_SWAPS)
    assert sw.rewrite_stats.tensors_swapped > 0
    for enc, dec in ((0, 0), (128, 128), (7, 3), (4096, 4096), (1, 0), (0, 1)):
        sw.ex.set_swap_grid(enc, dec)
        ls, st = sw.step()
        assert same_bits(lb, ls), (enc, dec)
        gs = sw.grad_bits()
        for k in gb:
            assert np.array_equal(gb[k], gs[k]), (enc, dec, k)
        assert st.bytes_d2h == st.bytes_h2d > 0
    for enc, dec in ((-1, 0), (0, 4097), (5000, 1)):
        with pytest.raises(L.LmsError) as e:
            sw.ex.set_swap_grid(enc, dec)
        assert e.value.status == A.EINVAL
    ls, _ = sw.step()                                 # a refused call changed nothing
    assert same_bits(lb, ls)
