"""Update phase on the GPU: several training steps in place, against the oracle's gradient descent."""
import numpy as np
import pytest

import workloads as W
from oracle import evaluate

pytestmark = pytest.mark.gpu

SPECS = {
    "tiny_chain": (lambda: W.tiny_chain(), 0.05),
    "pool_net": (lambda: W.pool_net(), 0.02),
    "updown_net": (lambda: W.updown_net(), 0.02),
    "resnet_small": (lambda: W.resnet50(batch=2, size=32, classes=10, stage_blocks=(1, 1, 1, 1), base=8), 0.02),
    # 71 parameters: the executor sends updates out in launches of up to 64, so this one needs two
    "resnet_71_parameters": (lambda: W.resnet50(batch=2, size=32, classes=10, stage_blocks=(2, 2, 1, 1), base=8), 0.02),
}
STEPS = 4


def rel(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-30)


@pytest.mark.parametrize("name", list(SPECS))
def test_fp32_training_follows_the_oracle(name):
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    make, lr = SPECS[name]
    spec = make()
    tensors = W.make_tensors(spec, affine="random")
    ref_losses, ref_params = evaluate.train_steps(spec, tensors, lr, STEPS)
    assert abs(ref_losses[-1] - ref_losses[0]) > 1e-3 * abs(ref_losses[0])      # the steps really move the loss
    s = Session(spec, tensors, dtype=A.F32, lr=lr)
    losses = [s.step()[0] for _ in range(STEPS)]
    print(name, losses, ref_losses)
    for a, b in zip(losses, ref_losses):
        assert abs(a - b) <= 1e-4 * abs(b)
    for k, v in ref_params.items():
        assert rel(s.param(k), v) <= 1e-4, k


@pytest.mark.parametrize("name", ["tiny_chain", "pool_net", "updown_net"])
def test_bf16_training_follows_the_quantised_oracle_and_swapping_changes_nothing(name):
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    make, lr = SPECS[name]
    spec = make()
    tensors = W.make_tensors(spec, affine="random")
    ref_losses, ref_params = evaluate.train_steps(spec, tensors, lr, STEPS, quant=True)
    s = Session(spec, tensors, lr=lr)
    losses = [s.step()[0] for _ in range(STEPS)]
    for a, b in zip(losses, ref_losses):
        assert abs(a - b) <= 1e-2 * abs(b)
    params = {k: s.param(k) for k in ref_params}
    for k, v in ref_params.items():
        assert rel(params[k], v) <= 1e-2, k
    del s
    # the rewritten graph trains bit-identically: swapped tensors, poison fill, encoded copies
    sw = Session(spec, tensors, lr=lr, rewrite=dict(fuse_swapins=1, lb=2), flags=A.X_POISON | A.X_ENCODE_SWAPS)
    assert sw.rewrite_stats.tensors_swapped > 0
    losses_sw = [sw.step()[0] for _ in range(STEPS)]
    assert [np.float32(x).view(np.uint32) for x in losses_sw] == [np.float32(x).view(np.uint32) for x in losses]
    for k in ref_params:
        assert np.array_equal(sw.param(k), params[k]), k


@pytest.mark.parametrize("name", ["tiny_chain", "pool_net", "updown_net"])
def test_momentum_training_follows_the_oracle(name):
    """Classical momentum (velocity variables updated in place next to the parameters): fp32 check mode against the
    exact oracle, bf16 against the oracle with bf16 storage, and a swapping run bit-identical to the plain one."""
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    make, lr = SPECS[name]
    spec = make()
    tensors = W.make_tensors(spec, affine="random")
    mu = 0.8
    ref_losses, ref_params = evaluate.train_steps(spec, tensors, lr, STEPS, momentum=mu)
    plain_losses, _ = evaluate.train_steps(spec, tensors, lr, STEPS)
    assert abs(ref_losses[-1] - plain_losses[-1]) > 1e-3 * abs(plain_losses[-1])     # momentum really changes the run
    s = Session(spec, tensors, dtype=A.F32, lr=lr, momentum=mu)
    names = [i.name.decode() for i in s.infos]
    assert any(n.startswith("velocity/") for n in names) and any(n.startswith("update/velocity/") for n in names)
    losses = [s.step()[0] for _ in range(STEPS)]
    for a, b in zip(losses, ref_losses):
        assert abs(a - b) <= 1e-4 * abs(b)
    for k, v in ref_params.items():
        assert rel(s.param(k), v) <= 1e-4, k
    del s
    q_losses, q_params = evaluate.train_steps(spec, tensors, lr, STEPS, quant=True, momentum=mu)
    b = Session(spec, tensors, lr=lr, momentum=mu)
    losses_b = [b.step()[0] for _ in range(STEPS)]
    for a, r in zip(losses_b, q_losses):
        assert abs(a - r) <= 1e-2 * abs(r)
    params_b = {k: b.param(k) for k in q_params}
    for k, v in q_params.items():
        assert rel(params_b[k], v) <= 1e-2, k
    del b
    sw = Session(spec, tensors, lr=lr, momentum=mu, rewrite=dict(fuse_swapins=1, lb=2), flags=A.X_POISON)
    assert sw.rewrite_stats.tensors_swapped > 0
    losses_sw = [sw.step()[0] for _ in range(STEPS)]
    assert [np.float32(x).view(np.uint32) for x in losses_sw] == [np.float32(x).view(np.uint32) for x in losses_b]
    for k in q_params:
        assert np.array_equal(sw.param(k), params_b[k]), k


def test_an_operation_reads_the_latest_value_of_a_variable():
    """Section 3.2: an operation always uses the latest value of a variable, and the variable comes first among the
    consumers of the tensor that updates it.  A second convolution with the same filter is created after the update
    operation of that filter: within the same step it must see w - lr * dw, not w."""
    import torch
    import paper_1807_02037_amd as L
    from oracle import ops
    A = L.abi
    lr = 0.25
    x = W.round_to_bf16(W.normal(4001, (2, 6, 6, 8)))
    w = W.round_to_bf16(W.normal(4002, (3, 3, 8, 8), 0.2))
    t = W.round_to_bf16(W.normal(4003, (2, 6, 6, 8)))
    g = L.Graph()
    xi = g.add_variable("x", A.F32, x.shape, A.VAR_INPUT)
    wi = g.add_variable("w", A.F32, w.shape, A.VAR_PARAM)
    ti = g.add_variable("t", A.F32, t.shape, A.VAR_TARGET)
    y1 = g.add_op("y1", A.OP_CONV, [xi, wi], stride=1, pad=1)
    loss = g.add_op("loss", A.OP_MSE, [y1, ti])
    g.build_backward(loss)
    assert g.build_update(lr) == 1
    y2 = g.add_op("y2", A.OP_CONV, [xi, wi], stride=1, pad=1)          # created after update/w
    names = {g.node_info(i).name.decode(): i for i in range(g.node_count())}
    upd, grad = names["update/w"], names["grad/w"]
    assert [(e.src, e.dst) for e in g.edges() if e.action == A.UPDATE] == [(upd, wi)]
    gam = g.topo_order()
    assert gam[wi] == 0 and gam[y2] == 1                                # the update edge raises no order (Definition 2)
    order = g.schedule()
    assert order.index(upd) < order.index(y2)
    need = sum((g.node_info(i).bytes + 255) // 256 * 256 + (g.node_info(i).workspace_bytes + 255) // 256 * 256
               for i in range(g.node_count()) if not g.node_info(i).is_variable)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda")
    streams = [torch.cuda.Stream() for _ in range(3)]
    ex = L.Executor(g, arena.data_ptr(), need, 0, 0, *[s.cuda_stream for s in streams], A.X_KEEP_ALL)
    dev = {k: torch.from_numpy(v.astype(np.float32)).cuda() for k, v in (("x", x), ("w", w), ("t", t))}
    y2_out = torch.zeros(x.shape[:-1] + (8,), dtype=torch.float32, device="cuda")
    dw = torch.zeros(w.shape, dtype=torch.float32, device="cuda")
    for name, buf in (("x", dev["x"]), ("w", dev["w"]), ("t", dev["t"]), ("update/w", dev["w"]), ("y2", y2_out), ("grad/w", dw)):
        ex.bind(names[name], buf.data_ptr())
    ex.step(True)
    torch.cuda.synchronize()
    y1_ref = ops.conv_fwd(x, w, 1, 1)
    dw_ref = ops.conv_wgrad(x, ops.mse_bwd(y1_ref, t), (3, 3), 1, 1)
    w_new = w - lr * dw_ref
    assert rel(dw.cpu().numpy().astype(np.float64), dw_ref) <= 1e-5
    assert rel(dev["w"].cpu().numpy().astype(np.float64), w_new) <= 1e-6
    got = y2_out.cpu().numpy().astype(np.float64)
    assert rel(got, ops.conv_fwd(x, w_new, 1, 1)) <= 1e-5
    assert rel(got, y1_ref) > 1e-2                                      # and not the value before the update


def test_rewritten_resnet_trains_bit_identically_with_the_hybrid_planner():
    """Update phase on a graph rewritten by the hybrid planner (swapped and recomputed tensors, weight-gradient nodes
    that wait for them): losses, every parameter and every gradient equal the plain run bit for bit over several
    steps.  The shift gradients come out of the weight-gradient passes, and the update operations read them."""
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    spec = W.resnet50(batch=8, size=64)
    tensors = W.make_tensors(spec, affine="random")
    base = Session(spec, tensors, lr=1e-2)
    floor = L.build_graph(spec)[0].rewrite(fuse_swapins=1, ctrld_strategy=A.OWN).arena_needed_after
    for frac in (0.25, 0.6):
        budget = int(floor + frac * (base.unswapped_need - floor))
        ref = Session(spec, tensors, lr=1e-2)
        sw = Session(spec, tensors, lr=1e-2, flags=A.X_ENCODE_SWAPS | A.X_POISON,
                     rewrite=dict(budget_bytes=budget, fuse_swapins=1, ctrld_strategy=A.OWN, recompute=2, encoded_swaps=1))
        assert sw.rewrite_stats.recomputed > 0
        for step in range(3):
            la, lb = ref.step()[0], sw.step()[0]
            assert np.float32(la).view(np.uint32) == np.float32(lb).view(np.uint32), (frac, step)
            ga, gb = ref.grad_bits(), sw.grad_bits()
            for k in ga:
                assert np.array_equal(ga[k], gb[k]), (frac, step, k)
            for k, t in ref.dev.items():
                if not k.startswith("grad/") and t.dtype != torch_int32():
                    assert np.array_equal(ref.param(k), sw.param(k)), (frac, step, k)


def torch_int32():
    import torch
    return torch.int32


def test_every_update_is_the_fused_multiply_add_of_its_gradient():
    """One step of a network with 71 parameters (two launches of batched updates, fp32 and bf16 tensors, sizes that
    are no multiple of the work-group): every element of every parameter is p - lr * g rounded once to fp32 (and then
    to nearest-even bf16 for bf16 parameters), with the gradient the same step reports."""
    from paper_1807_02037_amd.session import Session
    spec = W.resnet50(batch=2, size=32, classes=10, stage_blocks=(2, 2, 1, 1), base=8)
    tensors = W.make_tensors(spec, affine="random")
    lr = 0.02
    s = Session(spec, tensors, lr=lr)
    names = [k[len("grad/"):] for k in s.grads()]
    assert len(names) == 71
    before = {k: s.param(k) for k in names}
    s.step()
    grads = s.grads()
    checked = moved = 0
    for k in names:
        # the product of two fp32 numbers is exact in fp64, the sum is rounded to 53 bits and then to 24
        want = (before[k] - np.float64(np.float32(lr)) * grads["grad/" + k]).astype(np.float32)
        if s.dev[k].dtype.itemsize == 2:
            u = want.view(np.uint32).astype(np.uint64)
            want = (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16).astype(np.uint32).view(np.float32)
        got = s.param(k).astype(np.float32)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), k
        moved += not np.array_equal(got, before[k].astype(np.float32))
        checked += got.size
    assert checked > 10000 and moved >= 60          # the updates moved the parameters
