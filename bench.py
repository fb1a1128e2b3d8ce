"""Benchmark of the swap-rewritten CNN training step on one MI355X.

One step = one forward + backward pass of the whole rewritten graph (all convolution kernels,
loss, swap-out and swap-in copies) over one seeded synthetic batch that is already resident in
HBM.  Workload: the ResNet-50 conv2_x stage (3 bottleneck blocks, batch 64, 56x56x256, bf16)
with the device budget capped at half of the unswapped arena footprint.

Prints one JSON line: training samples/s, plus the roofline position of the dominant convolution
kernel (timed with events on the stream it is launched on) and the fp64 CPU oracle timed on a
bounded sample of the same workload.
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
PCIE_GEN5_X16_GBS = 63.0


def timed_steps(sess, steps, warmup):
    import torch
    for _ in range(warmup):
        sess.step(sync=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps - 1):
        sess.step(sync=False)
    loss, st = sess.step(sync=True)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3, loss, st


def calibration_copy(reps=10, mib=256):
    """A plain device-to-device copy of known size through the library's copy kernel: the reference that
    the HBM traffic counters of a profiler run are scaled by."""
    import ctypes
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


def kernel_rooflines(spec, reps=20):
    """Times every distinct convolution launch of the workload through the stand-alone C-ABI
    entry points, with events on the launch stream.  Returns a list of dicts."""
    import numpy as np
    import torch
    import paper_1807_02037_amd as L
    import workloads as W
    A = L.abi
    shp = W.infer_shapes(spec)
    stream = torch.cuda.current_stream()
    seen, out = set(), []
    first = True
    for Lr in spec["layers"]:
        if Lr["op"] != "conv":
            continue
        xs, ys = shp["act"][Lr["in"]], shp["act"][Lr["name"]]
        key = (xs, ys, Lr["filt"], Lr["stride"], Lr["pad"], Lr["res"] is not None)
        count_key = key
        if key in seen:
            for o in out:
                if o["key"] == str(count_key):
                    o["launches_per_step"] += 1
            continue
        is_first = first
        first = False
        seen.add(key)
        n, in_sp, c, k = xs[0], xs[1:-1], xs[-1], ys[-1]
        d = L.conv_desc(n, in_sp, c, k, Lr["filt"], Lr["stride"], Lr["pad"], A.F_RELU if Lr["relu"] else 0)
        x = torch.randn(xs, device="cuda").to(torch.bfloat16)
        w = (torch.randn(tuple(Lr["filt"]) + (c, k), device="cuda") * 0.05).to(torch.bfloat16)
        y = torch.empty(ys, device="cuda", dtype=torch.bfloat16)
        dy = torch.randn(ys, device="cuda").to(torch.bfloat16)
        dx = torch.empty(xs, device="cuda", dtype=torch.bfloat16)
        res = torch.randn(ys, device="cuda").to(torch.bfloat16) if Lr["res"] is not None else None
        dw = torch.empty(tuple(Lr["filt"]) + (c, k), device="cuda", dtype=torch.float32)
        wsb = max(L.conv_workspace_bytes(d, w_) for w_ in (A.CONV_FWD, A.CONV_DGRAD, A.CONV_WGRAD))
        ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
        nx, ny, nw = x.numel() * 2, y.numel() * 2, w.numel() * 2
        flops = 2.0 * y.numel() * c * int(np.prod(Lr["filt"]))
        calls = {
            "fwd": (lambda: L.conv_fwd(d, x.data_ptr(), w.data_ptr(), None, None, res.data_ptr() if res is not None else None,
                                       y.data_ptr(), ws.data_ptr(), stream.cuda_stream), nx + nw + ny + (ny if res is not None else 0)),
            "dgrad": (lambda: L.conv_dgrad(d, dy.data_ptr(), w.data_ptr(), None, None, x.data_ptr(), dx.data_ptr(), ws.data_ptr(),
                                           stream.cuda_stream), ny + nw + nx + nx),
            "wgrad": (lambda: L.conv_wgrad(d, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), ws.data_ptr(), stream.cuda_stream),
                      nx + ny + 2 * nw),
        }
        for which, (fn, nbytes) in calls.items():
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            e1.synchronize()
            ms = e0.elapsed_time(e1) / reps
            out.append({"key": str(count_key), "kernel": f"conv_{which} {xs}->{ys} filt{tuple(Lr['filt'])}",
                        "ms": ms, "bytes": nbytes, "flops": flops, "gbs": nbytes / ms / 1e6, "tflops": flops / ms / 1e9,
                        # the first layer has no data gradient: the input batch is not learnable
                        "launches_per_step": 0 if (which == "dgrad" and is_first) else 1})
    return out


def cpu_baseline(sample_batch=32, min_seconds=10.0):
    """The fp64 oracle on a bounded sample of the workload: whole passes over a batch-32 slice of the same
    stage, repeated until at least `min_seconds` of CPU work have been timed."""
    import workloads as W
    from oracle import evaluate
    spec = W.bottleneck_stage(batch=sample_batch)
    tensors = W.make_tensors(spec)
    passes, dt = 0, 0.0
    t0 = time.perf_counter()
    while dt < min_seconds and passes < 8:
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
            "sample": f"{passes} fp64 forward+backward passes of the same 3-block stage on batch {sample_batch} of 64 "
                      f"(56x56x256), {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--roofline-only", action="store_true",
                    help="only the per-kernel timing loops and the calibration copy (the command profiled for profiles/)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads as W
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    spec = W.bottleneck_stage()
    batch = spec["input"][1][0]
    if args.roofline_only:
        kern = kernel_rooflines(spec)
        print(json.dumps({"kernels": [{k: kd[k] for k in ("kernel", "ms", "bytes", "gbs", "tflops")} for kd in kern],
                          "calibration_copy": calibration_copy()}))
        return
    tensors = W.make_tensors(spec)

    # unconstrained reference run (no budget, no swapping)
    base = Session(spec, tensors)
    base_ms, base_loss, _ = timed_steps(base, args.steps, args.warmup)
    footprint = base.unswapped_need
    del base
    torch.cuda.empty_cache()

    budget = footprint // 2
    rw = dict(budget_bytes=budget, fuse_swapins=1, ctrld_strategy=A.OWN)
    # the timed configuration: swapped tensors cross the host link encoded (bitmap + non-zero elements, lossless)
    sess = Session(spec, tensors, rewrite=rw, flags=A.X_ENCODE_SWAPS)
    ms, loss, st = timed_steps(sess, args.steps, args.warmup)
    rs = sess.rewrite_stats
    assert sess.arena_bytes <= budget
    bit_exact = bool(abs(loss - base_loss) == 0.0)
    del sess
    torch.cuda.empty_cache()

    # the same plan with plain copies (swap-out and swap-in as two identities), overlapped and serial
    plain = Session(spec, tensors, rewrite=rw)
    plain_ms, plain_loss, plain_st = timed_steps(plain, max(3, args.steps // 2), 2)
    del plain
    torch.cuda.empty_cache()
    serial = Session(spec, tensors, rewrite=rw, flags=A.X_NO_OVERLAP)
    serial_ms, _, _ = timed_steps(serial, max(3, args.steps // 4), 1)
    del serial
    torch.cuda.empty_cache()

    kern = kernel_rooflines(spec)
    for kd in kern:
        kd["step_ms"] = kd["ms"] * kd["launches_per_step"]
    dom = max(kern, key=lambda kd: kd["step_ms"])
    conv_flops = sum(kd["flops"] * kd["launches_per_step"] for kd in kern)
    conv_ms = sum(kd["step_ms"] for kd in kern)

    copy_ms = max(serial_ms - base_ms, 1e-6)
    swap_bytes = plain_st.bytes_d2h + plain_st.bytes_h2d
    moved = st.bytes_d2h + st.bytes_h2d
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "dominant_kernel_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath)).get("per_call", {})
        if dom["kernel"] in tj:
            traffic = tj[dom["kernel"]].get("hbm_bytes_per_launch")
    result = {
        "metric": "train samples/s at max batch under HBM cap; conv MFMA util %; swap GB/s",
        "value": batch / (ms / 1e3),
        "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "ResNet-50 conv2_x stage, 3 bottleneck blocks, batch 64, 56x56x256, MSE; "
                               "HBM budget = half of the unswapped arena footprint",
                   "global_batch": batch, "budget_bytes": int(budget), "unswapped_footprint_bytes": int(footprint),
                   "tensors_swapped": rs.tensors_swapped, "swap_outs": rs.swap_outs, "swap_ins": rs.swap_ins,
                   "strategy": "own (hoist within budget), fused swap-ins, encoded swap copies"},
        "roofline": {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": dom["gbs"] / HBM_PEAK_GBS, "traffic": traffic, "ms": dom["ms"],
                     "algorithmic_bytes": dom["bytes"]},
        "unswapped": {"ms_per_step": base_ms, "samples_per_s": batch / (base_ms / 1e3)},
        "swap": {"tensor_bytes_each_way": int(plain_st.bytes_d2h),
                 "bytes_d2h": int(st.bytes_d2h), "bytes_h2d": int(st.bytes_h2d),
                 "encoded_fraction": moved / max(swap_bytes, 1),
                 "overhead_vs_unswapped": ms / base_ms - 1.0,
                 "plain_copies_ms_per_step": plain_ms, "plain_copies_serial_ms_per_step": serial_ms,
                 "copy_gbs_both_directions_serial": swap_bytes / copy_ms / 1e6,
                 "pcie_gen5_x16_peak_gbs_per_direction": PCIE_GEN5_X16_GBS,
                 # swap-outs can only hide under the forward pass and swap-ins under the backward pass
                 "swap_roofline_ms": max(base_ms, moved / PCIE_GEN5_X16_GBS / 1e6),
                 "frac_of_swap_roofline": max(base_ms, moved / PCIE_GEN5_X16_GBS / 1e6) / ms,
                 "link_gbs_while_swapping": moved / max(ms - base_ms, 1e-6) / 1e6,
                 "loss_bit_exact_vs_unswapped": bit_exact and bool(abs(plain_loss - base_loss) == 0.0)},
        "conv": {"mfma_util_vs_bf16_peak": conv_flops / (conv_ms / 1e3) / 2.5e15, "conv_kernel_ms_per_step": conv_ms,
                 "kernels": [{k: kd[k] for k in ("kernel", "ms", "gbs", "tflops", "launches_per_step")} for kd in kern]},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
