"""Benchmark of the swap-rewritten CNN training step on one MI355X.

One step = one forward + backward pass of the whole rewritten graph (all convolution kernels, loss, swap-out and
swap-in copies) over one seeded synthetic batch that is already resident in HBM.

Default run (`python bench.py`): the headline workload is ResNet-50 (per-channel affine in place of batch norm) at
224x224 under a 16 GB device arena, at the largest batch for which a rewritten plan fits the arena: the experiment of
Table 3 / Section 6 of the paper on synthetic inputs of the same shapes.  `value` = images/s of that swapping step.
Beside it: the largest batch that fits without swapping and its rate, the same large batch without a cap, plain
(unencoded) swap copies, link GB/s and the swap roofline; the roofline position of the dominant convolution launch
of the headline step (the most expensive geometry of the kernel family with the largest share of the step, timed
stand-alone with events on its launch stream); the fp64 CPU oracle timed on a bounded
sample; and short runs of the other configured workloads (ResNet-50 conv2_x stage at half its footprint, 3D U-Net
128^3 and 192^3) as extra keys.

Other modes (one JSON line per run):
    python bench.py --config resnet [--cap-gb 16] [--multipliers 1,1.5,2,3,4] [--plain-copies] [--recompute 0|1|2]
    python bench.py --config unet --size 192 --batch 1 [--fractions 0.5,0.25] [--recompute 0|1|2]
    python bench.py --config stage
    python bench.py --config sweep-resnet --batch 1276        (Table 2's parameters one at a time)
    python bench.py --config sweep-unet --size 192 --batch 1
    python bench.py --config sweep-resnet --at-largest-batch  (every setting at the largest batch it fits under the cap)
    python bench.py --roofline-only                            (dominant launch + calibration copy: the profiled command)

Large batches never exist as host arrays: the seeded tensors of the workload at a small batch are repeated along the
batch axis on the device (values do not influence timing).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
PCIE_GEN5_X16_GBS = 63.0
GB = 1e9
STAGED_SWAPS = "auto"    # set from --staged-swaps
METRIC = "train samples/s at max batch under HBM cap; conv MFMA util %; swap GB/s"


# ------------------------------------------------------------------------------------------------ helpers
# Learning rate of the update phase (Section 3.3) that every timed step ends with: plain gradient descent on all
# parameters, so a step is a whole training iteration.  Small, so that the activations of the timed steps keep the
# statistics of the first one.  None: no update phase.
LR = 1e-4


def first_losses(sess):
    """Two synchronised steps before anything is timed: the loss of the first depends on the forward pass alone, the
    loss of the second on every parameter gradient of the first as well (through the update phase).  Equal bits in two
    runs of the same batch say that the rewritten step computes what the plain one does."""
    return [sess.step(sync=True)[0] for _ in range(2)]


def timed_steps(sess, steps, warmup):
    import torch
    for i in range(warmup):
        sess.step(sync=(i == 0))       # a synchronised step first: staged swaps take their widths from it
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps - 1):
        sess.step(sync=False)
    loss, st = sess.step(sync=True)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3, loss, st


def release_memory():
    """Returns cached device memory and cached pinned host memory to the system: the next run's arena and pinned pool
    may be larger than any block the caches hold."""
    import torch
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()


def same_bits(a, b):
    import numpy as np
    return bool(np.float32(a).view(np.uint32) == np.float32(b).view(np.uint32))


def conv_flops_per_step(spec):
    """Multiply-add work of one forward + backward pass: 2*M*K*C*taps per pass, three passes per convolution
    (no data gradient for layers that read the input batch)."""
    import numpy as np
    import workloads as W
    shp = W.infer_shapes(spec)
    total = 0.0
    for L in spec["layers"]:
        if L["op"] not in ("conv", "tconv"):
            continue
        ys = shp["act"][L["name"]]
        xs = shp["act"][L["in"]]
        taps = int(np.prod(L["filt"])) if L["op"] == "conv" else 1
        f = 2.0 * float(np.prod(ys[:-1])) * ys[-1] * xs[-1] * taps
        total += f * (2 if L["in"] == spec["input"][0] else 3)
    return total


def device_tensors(spec, small_batch):
    """Seeded tensors at `small_batch`, repeated on the device to the batch of `spec`."""
    import numpy as np
    import torch
    import workloads as W
    from paper_1807_02037_amd import abi as A
    from paper_1807_02037_amd.models import build_graph
    batch = spec["input"][1][0]
    builder = W.resnet50 if spec["name"].startswith("resnet") else W.unet3d
    small = builder(batch=small_batch, size=spec["input"][1][1])
    host = W.make_tensors(small, affine="random" if spec["name"].startswith("resnet") else "unit")
    out = {}
    g, _ = build_graph(spec, backward=False)
    infos = {g.node_info(i).name.decode(): g.node_info(i) for i in range(g.node_count())}
    for name, arr in host.items():
        info = infos[name]
        want = tuple(info.dims[i] for i in range(info.ndim))
        if tuple(arr.shape) == want:
            out[name] = arr
            continue
        assert arr.shape[0] == small_batch and want[0] == batch and tuple(arr.shape[1:]) == want[1:], (name, arr.shape, want)
        dt = {A.BF16: torch.bfloat16, A.F32: torch.float32}.get(info.dtype, torch.int32)
        t = torch.from_numpy(np.ascontiguousarray(arr, dtype=np.int32 if dt == torch.int32 else np.float32)).to(dt).cuda()
        reps = (batch + small_batch - 1) // small_batch
        out[name] = t.repeat((reps,) + (1,) * (t.dim() - 1))[:batch].contiguous()
    return out


def largest_unswapped_batch(cap, size, make_spec=None):
    """Largest batch whose unswapped plan fits the cap (0 if not even one sample does).  make_spec(batch): the
    workload, ResNet-50 at size x size by default."""
    import workloads as W
    from paper_1807_02037_amd.models import build_graph
    make_spec = make_spec or (lambda b: W.resnet50(batch=b, size=size))
    lo, hi = 1, 2
    need = lambda b: build_graph(make_spec(b))[0].memory_need()[1]
    if need(1) > cap:
        return 0
    while need(hi) <= cap:
        lo, hi = hi, hi * 2
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if need(mid) <= cap:
            lo = mid
        else:
            hi = mid
    return lo


def largest_swapped_batch(cap, size, lo, rewrite_kw, make_spec=None):
    """Largest batch for which a rewritten plan fits the cap (the rewriter reports an infeasible budget).  With
    staged swaps the staging buffers are part of the cap."""
    import workloads as W
    import paper_1807_02037_amd as L
    if STAGED_SWAPS == 1:
        cap = cap - L.swap_staging_bytes()
    from paper_1807_02037_amd.api import LmsError
    from paper_1807_02037_amd.models import build_graph
    make_spec = make_spec or (lambda b: W.resnet50(batch=b, size=size))

    def fits(b):
        g = build_graph(make_spec(b))[0]
        try:
            g.rewrite(budget_bytes=cap, **rewrite_kw)
            return True
        except LmsError:
            return False
    lo = max(lo, 1)
    if not fits(lo):
        return 0
    hi = lo * 2
    while fits(hi):
        lo, hi = hi, hi * 2
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if fits(mid):
            lo = mid
        else:
            hi = mid
    return lo


def largest_batch_with_setting(cap, make_spec, kw, limit=1 << 16):
    """Largest batch whose plan, rewritten with the fixed tuning parameters kw, needs an arena of at most cap bytes (the
    paper's 'maximum batch size' of a setting, Section 6.2); planner work only.  A setting that carries a budget is
    given the cap as its budget instead."""
    from paper_1807_02037_amd.api import LmsError
    from paper_1807_02037_amd.models import build_graph
    kw = dict(kw)
    budgeted = kw.pop("budget_bytes", None) is not None

    def fits(b):
        g = build_graph(make_spec(b))[0]
        try:
            g.rewrite(budget_bytes=int(cap), **kw) if budgeted else g.rewrite(**kw)
        except LmsError:
            return False
        return g.memory_need()[1] <= cap
    if not fits(1):
        return 0
    lo, hi = 1, 2
    while hi <= limit and fits(hi):
        lo, hi = hi, hi * 2
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if fits(mid):
            lo = mid
        else:
            hi = mid
    return lo


def rewrite_kw(recompute=0, encoded=True):
    """Budget-driven selection and placement with fused swap-ins; recompute: 0 swaps alone, 2 the hybrid planner
    (per tensor recompute / swap / keep).  encoded: the swap copies will be encoded, which the planner's estimate of
    the bytes on the link takes into account."""
    from paper_1807_02037_amd import abi as A
    return dict(fuse_swapins=1, ctrld_strategy=A.OWN, recompute=int(recompute), encoded_swaps=int(bool(encoded)))


def stats_dict(st):
    return {k: (float(getattr(st, k)) if k.endswith("ms") else int(getattr(st, k))) for k, _ in st._fields_}


def run_uncapped(spec, tensors, steps, warmup):
    from paper_1807_02037_amd.session import Session
    batch = spec["input"][1][0]
    flops = conv_flops_per_step(spec)
    base = Session(spec, tensors, lr=LR)
    loss = first_losses(base)
    ms, _, _ = timed_steps(base, steps, warmup)
    footprint = base.unswapped_need
    del base
    release_memory()
    return {"ms_per_step": ms, "samples_per_s": batch / ms * 1e3, "conv_tflops": flops / ms / 1e9,
            "mfma_util_vs_bf16_peak": flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, "unswapped_footprint_bytes": int(footprint),
            "loss": loss}


def quick_step_ms(spec, tensors, budget, flags, recompute, staged):
    """Step time of the rewritten run with direct or staged swap copies from two steps after a synchronised one (which
    gives the staged copies their widths); None if the plan does not fit without the staging buffers' share."""
    import torch
    from paper_1807_02037_amd import abi as A
    from paper_1807_02037_amd.api import LmsError
    from paper_1807_02037_amd.session import Session
    import paper_1807_02037_amd as L
    rk = rewrite_kw(recompute, bool(flags & A.X_ENCODE_SWAPS))
    plan_budget = int(budget) - (L.swap_staging_bytes() if staged else 0)
    try:
        sess = Session(spec, tensors, rewrite=dict(budget_bytes=plan_budget, **rk), flags=flags | (A.X_STAGED_SWAPS if staged else 0),
                       arena_bytes=int(budget), lr=LR)
    except LmsError:
        return None
    sess.step(sync=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    sess.step(sync=False)
    sess.step(sync=True)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / 2 * 1e3
    swaps = sess.rewrite_stats.swap_outs
    del sess
    release_memory()
    return ms if swaps > 0 or not staged else None


def run_capped(spec, tensors, budget, steps, warmup, flags, base, recompute=0, timing=True):
    """The run rewritten for `budget` bytes; base: the dict run_uncapped returned for the same batch.  timing: one more
    step of the same plan with the executor's stream timing on (stall of the compute stream, busy time of the copy
    streams), outside the timed steps."""
    from paper_1807_02037_amd import abi as A
    from paper_1807_02037_amd.session import Session
    import paper_1807_02037_amd as L
    batch = spec["input"][1][0]
    plan_budget = int(budget)
    rk = rewrite_kw(recompute, bool(flags & A.X_ENCODE_SWAPS))
    staged = False
    if flags & A.X_ENCODE_SWAPS:
        if STAGED_SWAPS == "auto":
            # Staged swaps (copy engines) leave the convolutions undisturbed but move a few percent more bytes, and
            # their buffers take 143 MB of the budget, for which the planner may swap or recompute more: which of the
            # two gives the shorter step is measured, two steps each.  A small budget cannot spare the buffers.
            if L.swap_staging_bytes() <= 0.03 * plan_budget:
                t_staged = quick_step_ms(spec, tensors, budget, flags, recompute, True)
                if t_staged is not None:
                    t_direct = quick_step_ms(spec, tensors, budget, flags, recompute, False)
                    staged = t_direct is None or t_staged < 0.98 * t_direct
        else:
            staged = bool(STAGED_SWAPS) and 2 * L.swap_staging_bytes() <= plan_budget     # a small budget cannot spare the buffers
    if staged:
        # the staging buffers of the copy-engine transfers are part of the arena: the plan gets the rest
        flags |= A.X_STAGED_SWAPS
        plan_budget -= L.swap_staging_bytes()
    # the arena is the whole cap: what the plan does not need lets the planner keep fresh outputs away from blocks
    # whose swap-out is still running
    sess = Session(spec, tensors, rewrite=dict(budget_bytes=plan_budget, **rk), flags=flags, arena_bytes=int(budget), lr=LR)
    assert sess.arena_bytes <= budget
    loss = first_losses(sess)
    encode_wgs = None
    if (flags & A.X_ENCODE_SWAPS) and not staged and sess.rewrite_stats.swap_outs > 0:
        # The encoder saturates the host link with 512 work-groups and then slows the convolutions beside it; with 128
        # it leaves them alone and is 15 % slower itself.  Which gives the shorter step depends on whether the forward
        # phase is as long as its swap-outs: two untimed steps of each setting decide.
        import torch
        trial = {}
        for wgs in (512, 128):
            sess.ex.set_swap_grid(wgs, 0)
            sess.step(sync=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            sess.step(sync=False)
            sess.step(sync=True)
            torch.cuda.synchronize()
            trial[wgs] = time.perf_counter() - t0
        encode_wgs = 128 if trial[128] < 0.98 * trial[512] else 512
        sess.ex.set_swap_grid(encode_wgs, 0)
    ms, _, st = timed_steps(sess, steps, warmup)
    rs = sess.rewrite_stats
    moved = st.bytes_d2h + st.bytes_h2d
    roof = max(base["ms_per_step"], moved / PCIE_GEN5_X16_GBS / 1e6)
    out = {"ms_per_step": ms, "samples_per_s": batch / ms * 1e3, "tensors_swapped": rs.tensors_swapped,
           "swap_outs": rs.swap_outs, "swap_ins": rs.swap_ins, "recomputed": rs.recomputed,
           "encoded_copies": bool(flags & A.X_ENCODE_SWAPS), "staged_copies": staged, "encoder_workgroups": encode_wgs, "tensor_bytes_each_way": int(rs.swapped_bytes_out),
           "bytes_d2h": int(st.bytes_d2h), "bytes_h2d": int(st.bytes_h2d), "arena_bytes": int(sess.arena_bytes),
           "pinned_bytes": int(st.pinned_bytes_used),
           # caller memory bound to variables and parameter gradients: outside the arena, so outside the cap
           "bound_bytes_outside_arena": int(sum(t.numel() * t.element_size() for t in sess.dev.values())),
           "overhead_vs_uncapped": ms / base["ms_per_step"] - 1.0,
           # swap-outs hide under the forward pass and swap-ins under the backward pass of the same step
           "swap_roofline_ms": roof, "frac_of_swap_roofline": roof / ms,
           "link_gbs_while_swapping": moved / max(ms - base["ms_per_step"], 1e-6) / 1e6,
           "loss_bit_identical_to_uncapped": all(same_bits(a, b) for a, b in zip(loss, base["loss"])),
           "first_losses": [float(v) for v in loss], "first_losses_uncapped": [float(v) for v in base["loss"]],
           "step_stats": stats_dict(st)}
    del sess
    if timing:
        prof = Session(spec, tensors, rewrite=dict(budget_bytes=plan_budget, **rk), flags=flags | A.X_TIMING,
                       arena_bytes=int(budget), lr=LR)
        if encode_wgs:
            prof.ex.set_swap_grid(encode_wgs, 0)
        prof.step(sync=True)
        _, pst = prof.step(sync=True)
        out["stream_timing"] = {k: float(getattr(pst, k)) for k in ("ms", "device_ms", "stall_h2d_ms", "stall_d2h_ms",
                                                                    "busy_d2h_ms", "busy_h2d_ms")}
        out["stream_timing"]["d2h_gbs_while_busy"] = pst.bytes_d2h / max(pst.busy_d2h_ms, 1e-6) / 1e6
        out["stream_timing"]["h2d_gbs_while_busy"] = pst.bytes_h2d / max(pst.busy_h2d_ms, 1e-6) / 1e6
        del prof
    release_memory()
    return out


# ------------------------------------------------------------------------------------------------ kernels
def conv_launches(spec):
    """Distinct convolution geometries of a workload with their launch counts per step."""
    import workloads as W
    shp = W.infer_shapes(spec)
    seen = {}
    first = True
    for Lr in spec["layers"]:
        if Lr["op"] != "conv":
            continue
        xs, ys = shp["act"][Lr["in"]], shp["act"][Lr["name"]]
        key = (xs, ys, tuple(Lr["filt"]), Lr["stride"], Lr["pad"], Lr["res"] is not None, bool(Lr["affine"]), bool(Lr["relu"]))
        ent = seen.setdefault(key, {"xs": xs, "ys": ys, "L": Lr, "fwd": 0, "dgrad": 0, "wgrad": 0})
        ent["fwd"] += 1
        ent["wgrad"] += 1
        ent["dgrad"] += 0 if first else 1          # the first layer has no data gradient: the input batch is not learnable
        first = False
    return list(seen.values())


def launch_name(ent, which):
    Lr = ent["L"]
    res = " +residual" if which == "fwd" and Lr["res"] is not None else ""
    return f"conv_{which} {tuple(ent['xs'])}->{tuple(ent['ys'])} filt{tuple(Lr['filt'])} stride {Lr['stride']}{res}"


def time_conv_launch(ent, which, reps):
    """One convolution launch through the stand-alone C-ABI entry point, events on the launch stream."""
    import numpy as np
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    Lr, xs, ys = ent["L"], ent["xs"], ent["ys"]
    stream = torch.cuda.current_stream()
    n, in_sp, c, k = xs[0], xs[1:-1], xs[-1], ys[-1]
    d = L.conv_desc(n, in_sp, c, k, Lr["filt"], Lr["stride"], Lr["pad"], A.F_RELU if Lr["relu"] else 0)

    def rnd(shape, std=1.0):
        t = torch.empty(shape, device="cuda", dtype=torch.bfloat16)
        t.normal_(0.0, std)
        return t
    w = rnd(tuple(Lr["filt"]) + (c, k), 0.05)
    nx, ny, nw = int(np.prod(xs)) * 2, int(np.prod(ys)) * 2, w.numel() * 2
    wsb = L.conv_workspace_bytes(d, {"fwd": A.CONV_FWD, "dgrad": A.CONV_DGRAD, "wgrad": A.CONV_WGRAD}[which])
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    scale = shift = None
    if Lr["affine"]:
        scale = torch.ones(k, device="cuda", dtype=torch.float32)
        shift = torch.zeros(k, device="cuda", dtype=torch.float32)
    sp = stream.cuda_stream
    if which == "fwd":
        x, y = rnd(xs), torch.empty(ys, device="cuda", dtype=torch.bfloat16)
        res = rnd(ys) if Lr["res"] is not None else None
        fn = lambda: L.conv_fwd(d, x.data_ptr(), w.data_ptr(), scale.data_ptr() if scale is not None else None,
                                shift.data_ptr() if shift is not None else None, res.data_ptr() if res is not None else None,
                                y.data_ptr(), ws.data_ptr(), sp)
        nbytes = nx + nw + ny + (ny if res is not None else 0)
    elif which == "dgrad":
        dy, mask, dx = rnd(ys), rnd(xs), torch.empty(xs, device="cuda", dtype=torch.bfloat16)
        fn = lambda: L.conv_dgrad(d, dy.data_ptr(), w.data_ptr(), scale.data_ptr() if scale is not None else None, None,
                                  mask.data_ptr(), dx.data_ptr(), ws.data_ptr(), sp)
        nbytes = ny + nw + nx + nx                  # dy, filter, ReLU mask of the producer, dx
    else:
        x, dy = rnd(xs), rnd(ys)
        dw = torch.empty(tuple(Lr["filt"]) + (c, k), device="cuda", dtype=torch.float32)
        fn = lambda: L.conv_wgrad(d, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), ws.data_ptr(), sp)
        nbytes = nx + ny + 2 * nw                   # fp32 result
    for _ in range(2):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        fn()
    e1.record(stream)
    e1.synchronize()
    ms = e0.elapsed_time(e1) / reps
    flops = 2.0 * float(np.prod(ys)) * c * int(np.prod(Lr["filt"]))
    return {"kernel": launch_name(ent, which), "ms": ms, "bytes": nbytes, "flops": flops, "gbs": nbytes / ms / 1e6, "tflops": flops / ms / 1e9,
            "launches_per_step": ent[which]}


def kernel_rooflines(spec, reps=5, only=None):
    """Times every distinct convolution launch of the workload (or only the one named `only`)."""
    import torch
    out = []
    for ent in conv_launches(spec):
        for which in ("fwd", "dgrad", "wgrad"):
            if ent[which] == 0:
                continue
            if only is not None and only not in launch_name(ent, which):
                continue
            out.append(time_conv_launch(ent, which, reps))
            torch.cuda.empty_cache()
    for kd in out:
        kd["step_ms"] = kd["ms"] * kd["launches_per_step"]
    return out


def roofline_of(kd, traffic_path=os.path.join(ROOT, "profiles", "dominant_kernel_traffic.json")):
    """Roofline entry of one timed launch: against HBM if its arithmetic intensity is below the ridge
    (2.5 PFLOP/s / 8 TB/s = 312 flop/B), else against the bf16 MFMA peak."""
    ai = kd["flops"] / kd["bytes"]
    traffic = None
    if os.path.exists(traffic_path):
        tj = json.load(open(traffic_path)).get("per_call", {})
        if kd["kernel"] in tj:
            traffic = tj[kd["kernel"]].get("hbm_bytes_per_launch")
    if ai < MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS:
        return {"bound": "hbm", "kernel": kd["kernel"], "achieved": kd["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": kd["gbs"] / HBM_PEAK_GBS, "traffic": traffic, "ms": kd["ms"], "algorithmic_bytes": kd["bytes"],
                "launches_per_step": kd["launches_per_step"], "share_of_conv_time": kd.get("share"),
                "kernel_family": kd.get("family"), "family_share_of_conv_time": kd.get("family_share")}
    return {"bound": "mfma", "kernel": kd["kernel"], "achieved": kd["tflops"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": kd["tflops"] / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "ms": kd["ms"], "algorithmic_flops": kd["flops"],
            "launches_per_step": kd["launches_per_step"], "share_of_conv_time": kd.get("share"),
            "kernel_family": kd.get("family"), "family_share_of_conv_time": kd.get("family_share")}


def calibration_copy(reps=10, mib=256):
    """A plain device-to-device copy of known size through the library's copy kernel: the reference that
    the HBM traffic counters of a profiler run are scaled by."""
    import torch
    import paper_1807_02037_amd as L
    n = mib << 20
    a = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    fn = L.abi.lib().lms_device_copy
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn(b.data_ptr(), a.data_ptr(), n, stream.cuda_stream)
    e0.record(stream)
    for _ in range(reps):
        fn(b.data_ptr(), a.data_ptr(), n, stream.cuda_stream)
    e1.record(stream)
    e1.synchronize()
    ms = e0.elapsed_time(e1) / reps
    return {"bytes_read": n, "bytes_written": n, "ms": ms, "gbs": 2 * n / ms / 1e6}


def mfma_probe(iters=40000, reps=3):
    """The library's matrix-pipe probe (lms_mfma_probe): a stream of bf16 MFMAs with one LDS read per product and no
    global memory traffic, on operands of zeros and of random bfloat16 values.  The device lowers clock and issue rate
    with the switching activity of the operands, so the rate on random operands, not the data-sheet peak, is what a
    convolution on N(0,1) data can approach on this device; both are reported beside the peak."""
    import ctypes
    import torch
    import paper_1807_02037_amd as L
    fn = L.abi.lib().lms_mfma_probe
    stream = torch.cuda.current_stream()
    out = {}
    for name, rnd in (("zeros", 0), ("random", 1)):
        flops = ctypes.c_uint64(0)
        rc = fn(200, rnd, ctypes.byref(flops), stream.cuda_stream)
        assert rc == 0, rc
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            rc = fn(iters, rnd, ctypes.byref(flops), stream.cuda_stream)
            assert rc == 0, rc
        e1.record(stream)
        e1.synchronize()
        out[f"tflops_{name}_operands"] = flops.value * reps / e0.elapsed_time(e1) / 1e9
    out["what"] = "v_mfma_f32_32x32x16_bf16 stream with one 16-byte LDS read per product, 2 waves per SIMD, no global memory traffic"
    return out


def cpu_baseline(min_seconds=10.0, sample_batch=2, size=224):
    """The fp64 oracle on a bounded sample of the headline workload: whole forward + backward passes of the same
    ResNet-50 at 224x224 on `sample_batch` images, repeated until at least `min_seconds` of CPU work are timed."""
    import workloads as W
    from oracle import evaluate
    spec = W.resnet50(batch=sample_batch, size=size)
    tensors = W.make_tensors(spec, affine="random")
    passes, dt = 0, 0.0
    t0 = time.perf_counter()
    while dt < min_seconds and passes < 64:
        evaluate.train_step(spec, tensors)
        passes += 1
        dt = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env))
    return {"value": sample_batch * passes / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
            "sample": f"{passes} fp64 forward+backward passes of the same ResNet-50 ({size}x{size}) on a batch of "
                      f"{sample_batch} images, {dt:.1f} s (numpy, BLAS threads); per-image cost does not depend on the batch"}


# ------------------------------------------------------------------------------------------------ workloads
def headline_resnet(args):
    """ResNet-50 224x224 under a 16 GB arena at the largest batch a rewritten plan fits."""
    import torch
    import workloads as W
    from paper_1807_02037_amd import abi as A
    from paper_1807_02037_amd.api import LmsError
    size, cap = 224, int(args.cap_gb * GB)
    b0 = largest_unswapped_batch(cap, size)
    # the hybrid plan starts from the plan with swaps alone, so the largest batch is the same: search with that one
    global STAGED_SWAPS
    alternative = None
    if STAGED_SWAPS == "auto":
        # Direct or staged swap copies: the staging buffers are part of the cap, so the largest batch with them is a
        # little smaller.  Both are measured at their own largest batch (two steps each) and the higher rate is the
        # headline; the other one is reported beside it.
        rates = {}
        for mode in (0, 1):
            STAGED_SWAPS = mode
            bm = largest_swapped_batch(cap, size, b0, rewrite_kw(0))
            try:
                sp = W.resnet50(batch=bm, size=size)
                tn = device_tensors(sp, 8)
                ms = quick_step_ms(sp, tn, cap, A.X_ENCODE_SWAPS, args.recompute, bool(mode))
                del tn
            except (LmsError, RuntimeError):
                ms = None
            release_memory()
            if ms is not None:
                rates[mode] = {"staged_copies": bool(mode), "largest_batch": bm, "ms_per_step_two_steps": ms, "samples_per_s": bm / ms * 1e3}
        STAGED_SWAPS = max(rates, key=lambda m: rates[m]["samples_per_s"]) if rates else 0
        alternative = rates.get(1 - STAGED_SWAPS)
    bmax = largest_swapped_batch(cap, size, b0, rewrite_kw(0))
    # the unswapped limit: what the cap allows without the method
    spec0 = W.resnet50(batch=b0, size=size)
    base0 = run_uncapped(spec0, device_tensors(spec0, 8), args.steps, args.warmup)
    release_memory()
    batch, note, capped, base = bmax, "", None, None
    while capped is None:
        spec = W.resnet50(batch=batch, size=size)
        tensors = device_tensors(spec, 8)
        try:
            base = run_uncapped(spec, tensors, max(3, args.steps // 4), 2)
            capped = run_capped(spec, tensors, cap, args.steps, args.warmup, A.X_ENCODE_SWAPS, base, args.recompute)
        except (LmsError, RuntimeError) as e:       # pinned pool refused by the host: say so and take a smaller batch
            note += f"batch {batch} failed ({str(e)[:120]}); "
            del tensors
            release_memory()
            batch = int(batch * 0.85)
            if batch <= b0:
                raise
    plain = None
    if not args.no_extras:
        try:
            plain = run_capped(spec, tensors, cap, max(2, args.steps // 6), 1, 0, base, args.recompute)
        except (LmsError, RuntimeError) as e:
            plain = {"failed": str(e)[:160]}
    del tensors
    release_memory()
    kern = kernel_rooflines(spec, reps=3)
    conv_ms = sum(kd["step_ms"] for kd in kern)
    for kd in kern:
        kd["share"] = kd["step_ms"] / conv_ms
    # The dominant launch: no single geometry stands out (the largest take 4 % of the step each, and which of them is
    # largest changes from box to box), but the families of launches differ by a factor of two and more.  So: the
    # family with the largest share of the step, and its most expensive geometry.  A family is what the dispatch keys
    # on first: filter and stride, and whether positions are the rows of the product (forward and data gradient, which
    # is a forward convolution of the gradient with the transposed filter) or its reduction (weight gradient).
    family = lambda kd: ("conv_wgrad" if kd["kernel"].startswith("conv_wgrad") else "conv_fwd/dgrad") + " " + \
        kd["kernel"][kd["kernel"].index("filt"):].replace(" +residual", "")
    shares = {}
    for kd in kern:
        shares[family(kd)] = shares.get(family(kd), 0.0) + kd["step_ms"]
    top = max(shares, key=shares.get)
    dom = max((kd for kd in kern if family(kd) == top), key=lambda kd: kd["step_ms"])
    dom["family"], dom["family_share"] = top, shares[top] / conv_ms
    torch.cuda.empty_cache()
    copy = calibration_copy()
    result = {
        "metric": METRIC, "value": capped["samples_per_s"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": capped["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResNet-50 (affine for BN) {size}x{size}x3, 1000-way softmax cross-entropy, device arena capped at "
                               f"{args.cap_gb:g} GB, batch {batch} = largest batch a rewritten plan fits"
                               + ("" if batch == bmax else f" that the host could pin memory for (plan limit {bmax})")
                               + f" = {batch / b0:.2f}x the largest unswapped batch {b0}"
                               + (", swap copies through staging buffers inside the cap" if capped["staged_copies"] else ""),
                   "global_batch": batch, "budget_bytes": cap, "largest_unswapped_batch": b0, "largest_swapped_batch": bmax,
                   "tensors_swapped": capped["tensors_swapped"], "recomputed": capped["recomputed"],
                   "strategy": "budget-driven selection and swap-in placement, fused swap-ins, encoded swap copies"
                               + (", hybrid recompute / swap / keep planner" if args.recompute == 2 else ""),
                   "step": "forward, loss, backward" + (f", update of every parameter (gradient descent, lr {LR:g})" if LR else ""),
                   "outside_the_cap": "input batch, labels, weights and fp32 weight gradients are caller memory bound to the "
                                      f"executor, outside the arena: {capped['bound_bytes_outside_arena']} bytes",
                   "other_transfer": alternative,
                   "note": note},
        # copy_kernel_gbs: what this library's plain copy kernel (half reads, half writes) reaches on the same device,
        # measured in the same run: the practical ceiling for a kernel whose traffic is nearly half writes
        "roofline": {**roofline_of(dom), "copy_kernel_gbs": copy["gbs"]},
        "largest_unswapped": {"batch": b0, **{k: base0[k] for k in ("ms_per_step", "samples_per_s", "conv_tflops", "mfma_util_vs_bf16_peak")}},
        "same_batch_uncapped": {k: base[k] for k in ("ms_per_step", "samples_per_s", "conv_tflops", "mfma_util_vs_bf16_peak",
                                                     "unswapped_footprint_bytes")},
        "swap": {**capped, "pcie_gen5_x16_peak_gbs_per_direction": PCIE_GEN5_X16_GBS, "plain_copies": plain},
        "conv": {"mfma_util_vs_bf16_peak_conv_launches_only": sum(kd["flops"] * kd["launches_per_step"] for kd in kern) / conv_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                 "conv_kernel_ms_per_step": conv_ms,
                 "mfma_probe": mfma_probe(),
                 "top_kernels": [{k: kd[k] for k in ("kernel", "ms", "gbs", "tflops", "launches_per_step", "share")}
                                 for kd in sorted(kern, key=lambda kd: -kd["step_ms"])[:8]]},
    }
    return result


def stage_run(args, steps=None, warmup=None):
    """Config 2: ResNet-50 conv2_x stage, batch 64, budget = half of the unswapped footprint."""
    import workloads as W
    from paper_1807_02037_amd import abi as A
    steps, warmup = steps or args.steps, warmup or args.warmup
    spec = W.bottleneck_stage()
    tensors = W.make_tensors(spec)
    base = run_uncapped(spec, tensors, steps, warmup)
    budget = base["unswapped_footprint_bytes"] // 2
    out = {"workload": "ResNet-50 conv2_x stage, 3 bottleneck blocks, batch 64, 56x56x256, MSE; budget = half of the unswapped footprint",
           "uncapped": {k: v for k, v in base.items() if k != "loss"}}
    out["capped_encoded"] = run_capped(spec, tensors, budget, steps, warmup, A.X_ENCODE_SWAPS, base, args.recompute)
    out["capped_plain"] = run_capped(spec, tensors, budget, max(3, steps // 2), 2, 0, base, args.recompute)
    out["capped_encoded_swaps_alone"] = run_capped(spec, tensors, budget, max(3, steps // 2), 2, A.X_ENCODE_SWAPS, base, 0)
    return out


def unet_run(args, size, batch, fractions, steps=None, warmup=None):
    import workloads as W
    from paper_1807_02037_amd import abi as A
    from paper_1807_02037_amd.api import LmsError
    steps, warmup = steps or args.steps, warmup or args.warmup
    spec = W.unet3d(batch=batch, size=size)
    tensors = device_tensors(spec, 1)
    cap = int(args.cap_gb * GB)
    base = run_uncapped(spec, tensors, steps, warmup)
    fp = base["unswapped_footprint_bytes"]
    out = {"workload": f"3D U-Net {size}^3, batch {batch}", "uncapped": {k: v for k, v in base.items() if k != "loss"},
           f"capped_{args.cap_gb:g}gb": "fits without swapping" if fp <= cap else None}
    # the 3-D convolutions are bound by the matrix pipe: the whole step's convolution rate beside what the pipe gives
    # on random operands on this device (lms_mfma_probe)
    out["mfma_probe"] = mfma_probe()
    out["uncapped"]["conv_tflops_over_probe_random"] = base["conv_tflops"] / out["mfma_probe"]["tflops_random_operands"]
    flags = 0 if args.plain_copies else A.X_ENCODE_SWAPS
    budgets = ([] if fp <= cap else [(f"capped_{args.cap_gb:g}gb", cap)]) + [(f"capped_{f:g}_of_footprint", int(fp * f)) for f in fractions]
    if args.uncapped_only:
        budgets = []
    for key, budget in budgets:
        try:
            out[key] = run_capped(spec, tensors, budget, steps, warmup, flags, base, args.recompute)
        except LmsError as e:
            out[key] = "failed: " + str(e)[:200]
            release_memory()
    return out


def unet_max_batch(args):
    """Table 3's experiment on the 3D U-Net: the largest batch that fits the cap without swapping, the largest a
    rewritten plan fits, and both timed (the larger one also in an arena of its unswapped size, for the overhead)."""
    import workloads as W
    from paper_1807_02037_amd import abi as A
    size, cap = args.size or 192, int(args.cap_gb * GB)
    make = lambda b: W.unet3d(batch=b, size=size)
    b0 = largest_unswapped_batch(cap, size, make)
    bmax = largest_swapped_batch(cap, size, b0, rewrite_kw(0), make)
    out = {"workload": f"3D U-Net {size}^3", "cap_gb": args.cap_gb, "largest_unswapped_batch": b0, "largest_swapped_batch": bmax,
           "ratio": bmax / b0 if b0 else None}
    print(json.dumps(out), flush=True)
    flags = 0 if args.plain_copies else A.X_ENCODE_SWAPS
    for batch in sorted({b for b in (b0, bmax) if b > 0}):
        spec = make(batch)
        tensors = device_tensors(spec, 1)
        base = run_uncapped(spec, tensors, args.steps, args.warmup)
        r = {"workload": f"3D U-Net {size}^3", "batch": batch, "uncapped": {k: v for k, v in base.items() if k != "loss"}}
        if base["unswapped_footprint_bytes"] <= cap:
            r["capped"] = "fits without swapping"
        else:
            try:
                r["capped"] = run_capped(spec, tensors, cap, args.steps, args.warmup, flags, base, args.recompute)
            except Exception as e:
                r["capped"] = "failed: " + str(e)[:200]
        print(json.dumps(r), flush=True)
        del tensors
        release_memory()


def sweep_settings(spec):
    """The settings of the sweeps: Table 2's tuning parameters one at a time, then the budget-driven planner."""
    from paper_1807_02037_amd import abi as A
    from paper_1807_02037_amd.models import build_graph
    settings = []
    for strat in (A.CHAIN_RULE, A.DIRECT_ORDER):
        for lb in (1, 5, 20, 100):
            settings.append(dict(n_tensors=-1, lb=lb, ctrld_strategy=strat, fuse_swapins=1))
    g0 = build_graph(spec)[0]
    n_all = g0.rewrite(n_tensors=-1, fuse_swapins=1).tensors_swapped
    for n in sorted({max(1, n_all // 8), max(1, n_all // 4), max(1, n_all // 2), max(1, 3 * n_all // 4)}):
        settings.append(dict(n_tensors=n, lb=1, ctrld_strategy=A.CHAIN_RULE, fuse_swapins=1))
    settings.append(dict(n_tensors=-1, lb=1, ctrld_strategy=A.CHAIN_RULE, fuse_swapins=0))
    settings.append(dict(n_tensors=-1, lb=1, ctrld_strategy=A.CHAIN_RULE, fuse_swapins=1, swap_branches=1, branch_threshold=20))
    settings.append(dict(n_tensors=-1, lb=1, ctrld_strategy=A.CHAIN_RULE, fuse_swapins=1, swap_branches=1, branch_threshold=5))
    for n in sorted({max(1, n_all // 4), max(1, n_all // 2), n_all}):
        # budget-driven selection and placement: the budget is the arena that the chain-rule plan with n tensors needs
        g = build_graph(spec)[0]
        g.rewrite(n_tensors=n, lb=1, ctrld_strategy=A.CHAIN_RULE, fuse_swapins=1)
        settings.append(dict(ctrld_strategy=A.OWN, fuse_swapins=1, budget_bytes=int(g.memory_need()[1])))
    return settings


def run_setting(rec, spec, tensors, kw, flags, steps, warmup, base_loss):
    """One rewritten run of a sweep; fills rec."""
    from paper_1807_02037_amd.session import Session
    batch = spec["input"][1][0]
    try:
        sess = Session(spec, tensors, rewrite=kw, flags=flags, lr=LR)
        loss = first_losses(sess)
        ms, _, st = timed_steps(sess, steps, warmup)
        rs = sess.rewrite_stats
        rec.update({"arena_gb": sess.arena_bytes / GB, "tensors_swapped": rs.tensors_swapped, "swap_outs": rs.swap_outs,
                    "swap_ins": rs.swap_ins, "gb_out": st.bytes_d2h / GB, "gb_in": st.bytes_h2d / GB, "ms_per_step": ms,
                    "samples_per_s": batch / ms * 1e3, "step_stats": stats_dict(st),
                    "loss_bit_identical": all(same_bits(a, b) for a, b in zip(loss, base_loss))})
        del sess
    except Exception as e:
        rec["failed"] = str(e)[:160]
    release_memory()


def sweep(spec, tensors, label, steps, warmup, flags=0, make_spec=None, cap=None, at_largest=False, small_batch=1,
          which=None):
    """Table 2's tuning parameters one at a time (Section 5.2 / 6.2 of the paper): every setting is planned, run in an
    arena of exactly the size its plan needs, and reported as (arena needed, bytes swapped, step time); with
    make_spec(batch) and a cap, also the largest batch the setting fits under the cap (the planner alone).
    at_largest: every setting is run at that batch of its own instead of the batch of spec (the paper's Figures 4-7
    plot images/s against the batch per setting: this is each curve's last point)."""
    from paper_1807_02037_amd import abi as A
    from paper_1807_02037_amd.session import Session
    names = {A.CHAIN_RULE: "chain_rule", A.DIRECT_ORDER: "direct_order", A.OWN: "own"}
    show = lambda kw: {k: (names[v] if k == "ctrld_strategy" else v) for k, v in kw.items()}
    largest = (lambda kw: largest_batch_with_setting(cap, make_spec, kw)) if make_spec and cap else (lambda kw: None)
    settings = sweep_settings(spec)
    if which:                                      # "first:last" of the list, for a run in parts
        first, last = (int(v) if v else None for v in which.split(":"))
        settings = settings[first:last]

    def plain(spec_b, tensors_b):
        base = Session(spec_b, tensors_b, lr=LR)
        loss = first_losses(base)
        ms, _, _ = timed_steps(base, steps, warmup)
        arena = base.arena_bytes
        del base
        release_memory()
        return loss, ms, arena

    if at_largest:
        assert make_spec and cap
        seen, plain_runs = set(), {}
        for kw in settings:
            if "budget_bytes" in kw:
                kw = dict(kw, budget_bytes=int(cap))
            if json.dumps(show(kw), sort_keys=True) in seen:
                continue
            seen.add(json.dumps(show(kw), sort_keys=True))
            b = largest(kw)
            rec = {"workload": label, "batch": b, "setting": show(kw), "largest_batch_under_cap": b, "cap_gb": cap / GB}
            if b > 0:
                spec_b = make_spec(b)
                tensors_b = device_tensors(spec_b, min(small_batch, b))
                if b not in plain_runs:
                    plain_runs[b] = plain(spec_b, tensors_b)
                    print(json.dumps({"workload": label, "batch": b, "setting": "no rewriting", "arena_gb": plain_runs[b][2] / GB,
                                      "ms_per_step": plain_runs[b][1], "samples_per_s": b / plain_runs[b][1] * 1e3}), flush=True)
                run_setting(rec, spec_b, tensors_b, kw, flags, steps, warmup, plain_runs[b][0])
                del tensors_b
                release_memory()
            print(json.dumps(rec), flush=True)
        return
    batch = spec["input"][1][0]
    base_loss, base_ms, base_arena = plain(spec, tensors)
    print(json.dumps({"workload": label, "batch": batch, "setting": "no rewriting", "arena_gb": base_arena / GB,
                      "ms_per_step": base_ms, "samples_per_s": batch / base_ms * 1e3, "cap_gb": cap / GB if cap else None,
                      "largest_batch_under_cap": largest_unswapped_batch(cap, None, make_spec) if make_spec and cap else None}),
          flush=True)
    for kw in settings:
        rec = {"workload": label, "batch": batch, "setting": show(kw), "largest_batch_under_cap": largest(kw)}
        run_setting(rec, spec, tensors, kw, flags, steps, warmup, base_loss)
        print(json.dumps(rec), flush=True)


def flags_encode(args):
    return not (args.dma_copies or args.plain_copies)


def resnet_batches(args):
    """Batch sweep of config 3: B0 (largest unswapped batch) times each multiplier, and the largest swapped batch."""
    import workloads as W
    from paper_1807_02037_amd import abi as A
    size, cap = args.size or 224, int(args.cap_gb * GB)
    b0 = largest_unswapped_batch(cap, size)
    bmax = largest_swapped_batch(cap, size, b0, rewrite_kw(0))
    print(json.dumps({"workload": f"ResNet-50 {size}x{size}", "cap_gb": args.cap_gb, "largest_unswapped_batch": b0,
                      "largest_swapped_batch": bmax, "ratio": bmax / b0}), flush=True)
    mult = [float(v) for v in args.multipliers.split(",") if b0 * float(v) < bmax] + ([] if args.uncapped_only else [bmax / b0])
    if STAGED_SWAPS == "auto" and flags_encode(args) and not args.uncapped_only:
        # the largest batch that leaves room for the staging buffers of staged swap copies: a row of its own
        import paper_1807_02037_amd as L
        bst = largest_swapped_batch(cap - L.swap_staging_bytes(), size, b0, rewrite_kw(0))
        if b0 < bst < bmax:
            mult.insert(len(mult) - 1, bst / b0)
    if args.only_batch:
        mult = [args.only_batch / b0]
    flags = A.X_DMA_COPY if args.dma_copies else (0 if args.plain_copies else A.X_ENCODE_SWAPS)
    for m in mult:
        batch = int(round(b0 * m))
        spec = W.resnet50(batch=batch, size=size)
        tensors = device_tensors(spec, 8)
        base = run_uncapped(spec, tensors, args.steps, args.warmup)
        r = {"workload": f"ResNet-50 {size}x{size}", "batch": batch, "multiple_of_unswapped_batch": m,
             "uncapped": {k: v for k, v in base.items() if k != "loss"}}
        if base["unswapped_footprint_bytes"] <= cap:
            r["capped"] = "fits without swapping"
        elif args.uncapped_only:
            r["capped"] = "not run"
        else:
            try:
                r["capped"] = run_capped(spec, tensors, cap, args.steps, args.warmup, flags, base, args.recompute)
            except Exception as e:
                r["capped"] = "failed: " + str(e)[:200]
        print(json.dumps(r), flush=True)
        del tensors
        release_memory()


def main():
    global STAGED_SWAPS, LR
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="headline",
                    choices=["headline", "resnet", "stage", "unet", "unet-max", "sweep-resnet", "sweep-unet"])
    ap.add_argument("--cap-gb", type=float, default=16.0)
    ap.add_argument("--multipliers", default="1,1.5,2,3,4")
    ap.add_argument("--size", type=int, default=None)
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--fractions", default="0.5,0.25", help="unet: budgets as fractions of the unswapped footprint")
    ap.add_argument("--plain-copies", action="store_true",
                    help="swap-out / swap-in as two identities instead of the lossless encoding pair")
    ap.add_argument("--staged-swaps", default="auto", choices=["auto", "0", "1"],
                    help="encoded swap copies cross the link through the copy engines (LMS_X_STAGED_SWAPS): always, never, or "
                         "(default) where the plan's copies are short against the unswapped step")
    ap.add_argument("--dma-copies", action="store_true",
                    help="plain swap copies through hipMemcpyAsync (the copy engines) instead of the copy kernel")
    ap.add_argument("--recompute", type=int, default=2, choices=[0, 1, 2],
                    help="0: swaps alone; 1: cheap operations recomputed; 2 (default): hybrid planner, per tensor "
                         "recompute / swap / keep under the budget")
    ap.add_argument("--only-batch", type=int, default=0, help="resnet: this batch only, instead of the multiples of the unswapped batch")
    ap.add_argument("--uncapped-only", action="store_true",
                    help="resnet / unet: time the unswapped runs only (for a per-kernel profile of the plain step)")
    ap.add_argument("--at-largest-batch", action="store_true",
                    help="sweep-resnet / sweep-unet: run every setting at the largest batch it fits under the cap")
    ap.add_argument("--settings", default=None, help="sweeps: first:last of the list of settings (a sweep run in parts)")
    ap.add_argument("--lr", type=float, default=LR,
                    help="learning rate of the update phase every step ends with (plain gradient descent); 0: no update phase")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="headline only: skip the plain-copy run and the other workloads")
    ap.add_argument("--roofline-only", action="store_true",
                    help="only the dominant convolution launch of the headline step and the calibration copy "
                         "(the command profiled for profiles/)")
    ap.add_argument("--roofline-kernel", default=None,
                    help="with --roofline-only: only launches whose printed name contains this text")
    ap.add_argument("--roofline-batch", type=int, default=3796)
    ap.add_argument("--roofline-workload", default="resnet", choices=["resnet", "stage", "unet128", "unet192"],
                    help="with --roofline-only: the workload whose convolution launches are timed")
    args = ap.parse_args()
    STAGED_SWAPS = "auto" if args.staged_swaps == "auto" else int(args.staged_swaps)
    LR = args.lr if args.lr > 0 else None
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads as W
    from paper_1807_02037_amd import abi as A
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    if args.roofline_only:
        spec = {"resnet": lambda: W.resnet50(batch=args.roofline_batch, size=224), "stage": W.bottleneck_stage,
                "unet128": lambda: W.unet3d(batch=1, size=128), "unet192": lambda: W.unet3d(batch=1, size=192)}[args.roofline_workload]()
        kern = kernel_rooflines(spec, reps=10, only=args.roofline_kernel)
        print(json.dumps({"kernels": [{k: kd[k] for k in ("kernel", "ms", "bytes", "gbs", "tflops", "launches_per_step")} for kd in kern],
                          "calibration_copy": calibration_copy()}))
        return
    if args.config == "headline":
        mode = STAGED_SWAPS
        result = headline_resnet(args)
        STAGED_SWAPS = mode            # the headline fixed its own choice; the other workloads choose for themselves
        if not args.no_extras:
            short = dict(steps=max(5, args.steps // 2), warmup=2)
            result["other_configs"] = {"stage_batch64": stage_run(args, **short),
                                       "unet_128": unet_run(args, 128, 1, [0.5], **short),
                                       "unet_192": unet_run(args, 192, 1, [0.5], **short)}
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = cpu_baseline()
        print(json.dumps(result))
    elif args.config == "resnet":
        resnet_batches(args)
    elif args.config == "stage":
        print(json.dumps(stage_run(args)))
    elif args.config == "unet-max":
        unet_max_batch(args)
    elif args.config == "unet":
        fr = [float(v) for v in args.fractions.split(",") if v]
        print(json.dumps(unet_run(args, args.size or 128, args.batch, fr)))
    else:
        flags = 0 if args.plain_copies else A.X_ENCODE_SWAPS
        if args.config == "sweep-resnet":
            make_spec = lambda b: W.resnet50(batch=b, size=args.size or 224)
            spec = make_spec(args.batch)
            tensors, label = device_tensors(spec, 8), f"ResNet-50 {args.size or 224}x{args.size or 224}"
        else:
            make_spec = lambda b: W.unet3d(batch=b, size=args.size or 192)
            spec = make_spec(args.batch)
            tensors, label = device_tensors(spec, 1), f"3D U-Net {args.size or 192}^3"
        sweep(spec, tensors, label, args.steps, args.warmup, flags, make_spec, args.cap_gb * GB, args.at_largest_batch,
              8 if args.config == "sweep-resnet" else 1, args.settings)


if __name__ == "__main__":
    main()
