"""Throughput under a device-memory cap for the larger workloads (ResNet-50 at 224x224, 3D U-Net at 128^3
and 192^3): the measurements of the evaluation in Section 5 of the paper, on synthetic inputs of the same
shapes.  Prints one JSON line per run.

    python -m paper_1807_02037_amd.measure_configs resnet [--cap-gb 16] [--multipliers 1,1.5,2,3,4]
    python -m paper_1807_02037_amd.measure_configs unet --size 192 --batch 1 [--cap-gb 16]
    python -m paper_1807_02037_amd.measure_configs sweep-resnet --batch 1276
    python -m paper_1807_02037_amd.measure_configs sweep-unet --size 192 --batch 1

resnet: finds B0, the largest batch whose unswapped plan fits the cap, and the largest batch a rewritten plan fits, then runs B0 x multiplier (and the largest batch) with the
graph rewritten for the cap (smallest number of swapped tensors that fits, fused swap-ins, swap-ins hoisted
as far as the cap allows) and reports samples/s, swapped bytes and the overhead against an uncapped run of
the same batch.  Swapped tensors cross the host link in the lossless encoded form unless --plain-copies is given.  unet: one volume size and batch, capped at --cap-gb and at 1/2 and 1/4 of the unswapped
footprint, each compared with the uncapped run (loss must be bit-identical).  sweep-*: the tuning parameters of
Table 2 one at a time (n_tensors, lb, ctrld_strategy, fuse_swapins, swap_branches), each setting in an arena of exactly
the size its plan needs.

Inputs are the seeded synthetic tensors of the workload at a small batch, repeated along the batch axis on
the device: values do not influence timing and a large batch never exists as a host array.
"""
import argparse
import json
import sys
import time

import numpy as np
import torch

import workloads as W
from . import _lib as A
from .models import build_graph
from .session import Session

GB = 1e9


def conv_flops_per_step(spec):
    """Multiply-add work of one forward + backward pass: 2*M*K*C*taps per pass, three passes per convolution
    (no data gradient for layers that read the input batch)."""
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
    batch = spec["input"][1][0]
    small = dict(spec)
    builder = W.resnet50 if spec["name"].startswith("resnet") else W.unet3d
    small = builder(batch=small_batch, size=spec["input"][1][1])
    host = W.make_tensors(small, affine="random" if spec["name"].startswith("resnet") else "unit")
    big = W.infer_shapes(spec)
    out = {}
    g, _ = build_graph(spec)
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


def release_memory():
    """Returns cached device memory and cached pinned host memory to the system: the next run's arena and pinned pool
    may be larger than any block the caches hold."""
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()


def timed(sess, steps, warmup):
    for _ in range(warmup):
        sess.step(sync=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps - 1):
        sess.step(sync=False)
    loss, st = sess.step(sync=True)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3, loss, st


def run_pair(spec, tensors, budget, steps, warmup, label, flags=0, recompute=0, uncapped_only=False):
    """Uncapped run, then (unless uncapped_only) the run rewritten for `budget` bytes.  Returns a dict."""
    batch = spec["input"][1][0]
    flops = conv_flops_per_step(spec)
    base = Session(spec, tensors)
    base_ms, base_loss, _ = timed(base, steps, warmup)
    footprint = base.unswapped_need
    del base
    release_memory()
    out = {"workload": label, "batch": batch, "unswapped_footprint_gb": footprint / GB, "budget_gb": budget / GB,
           "uncapped": {"ms_per_step": base_ms, "samples_per_s": batch / base_ms * 1e3,
                        "conv_tflops": flops / base_ms / 1e9, "mfma_util_vs_bf16_peak": flops / base_ms / 1e9 / 2500.0}}
    if footprint <= budget:
        out["capped"] = "fits without swapping"
        return out
    if uncapped_only:
        out["capped"] = "not run"
        return out
    try:
        sess = Session(spec, tensors, rewrite=dict(budget_bytes=int(budget), fuse_swapins=1, ctrld_strategy=A.OWN, recompute=recompute),
                       flags=flags)
    except Exception as e:      # infeasible budget or host pool too large: report, do not raise the budget silently
        out["capped"] = "failed: " + str(e)[:200]
        return out
    assert sess.arena_bytes <= budget
    ms, loss, st = timed(sess, steps, warmup)
    rs = sess.rewrite_stats
    out["capped"] = {"ms_per_step": ms, "samples_per_s": batch / ms * 1e3, "tensors_swapped": rs.tensors_swapped,
                     "swap_outs": rs.swap_outs, "swap_ins": rs.swap_ins, "recomputed": rs.recomputed, "encoded_copies": bool(flags & A.X_ENCODE_SWAPS),
                     "tensor_gb_each_way": rs.swapped_bytes_out / GB, "bytes_d2h_gb": st.bytes_d2h / GB,
                     "bytes_h2d_gb": st.bytes_h2d / GB, "arena_gb": sess.arena_bytes / GB,
                     "overhead_vs_uncapped": ms / base_ms - 1.0,
                     "swap_roofline_ms": max(base_ms, (st.bytes_d2h + st.bytes_h2d) / 63e9 * 1e3),
                     "loss_bit_identical": bool(np.float32(loss).view(np.uint32) == np.float32(base_loss).view(np.uint32))}
    del sess
    release_memory()
    return out


def largest_unswapped_batch(cap, size):
    lo, hi = 1, 2
    need = lambda b: build_graph(W.resnet50(batch=b, size=size))[0].memory_need()[1]
    while need(hi) <= cap:
        lo, hi = hi, hi * 2
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if need(mid) <= cap:
            lo = mid
        else:
            hi = mid
    return lo


def largest_swapped_batch(cap, size, lo):
    """Largest batch for which a rewritten plan fits the cap (the rewriter reports an infeasible budget)."""
    from .api import LmsError

    def fits(b):
        g = build_graph(W.resnet50(batch=b, size=size))[0]
        try:
            g.rewrite(budget_bytes=cap, fuse_swapins=1, ctrld_strategy=A.OWN)
            return True
        except LmsError:
            return False
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


def sweep(spec, tensors, label, steps, warmup, flags=0):
    """Table 2's tuning parameters one at a time (Section 5.2 / 6.2 of the paper): every setting is planned, run in an
    arena of exactly the size its plan needs, and reported as (arena needed, bytes swapped, step time)."""
    batch = spec["input"][1][0]
    base = Session(spec, tensors)
    base_ms, base_loss, _ = timed(base, steps, warmup)
    print(json.dumps({"workload": label, "batch": batch, "setting": "no rewriting", "arena_gb": base.arena_bytes / GB,
                      "ms_per_step": base_ms, "samples_per_s": batch / base_ms * 1e3}), flush=True)
    del base
    release_memory()
    names = {A.CHAIN_RULE: "chain_rule", A.DIRECT_ORDER: "direct_order", A.OWN: "own"}
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
    for kw in settings:
        rec = {"workload": label, "batch": batch,
               "setting": {k: (names[v] if k == "ctrld_strategy" else v) for k, v in kw.items()}}
        try:
            sess = Session(spec, tensors, rewrite=kw, flags=flags)
            ms, loss, st = timed(sess, steps, warmup)
            rs = sess.rewrite_stats
            rec.update({"arena_gb": sess.arena_bytes / GB, "tensors_swapped": rs.tensors_swapped, "swap_outs": rs.swap_outs,
                        "swap_ins": rs.swap_ins, "gb_out": st.bytes_d2h / GB, "gb_in": st.bytes_h2d / GB, "ms_per_step": ms,
                        "samples_per_s": batch / ms * 1e3,
                        "loss_bit_identical": bool(np.float32(loss).view(np.uint32) == np.float32(base_loss).view(np.uint32))})
            del sess
        except Exception as e:
            rec["failed"] = str(e)[:160]
        release_memory()
        print(json.dumps(rec), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("which", choices=["resnet", "unet", "sweep-resnet", "sweep-unet"])
    ap.add_argument("--cap-gb", type=float, default=16.0)
    ap.add_argument("--multipliers", default="1,1.5,2,3,4")
    ap.add_argument("--size", type=int, default=None)
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--plain-copies", action="store_true",
                    help="swap-out / swap-in as two identities instead of the lossless encoding pair")
    ap.add_argument("--fractions", default="0.5,0.25", help="unet: budgets as fractions of the unswapped footprint")
    ap.add_argument("--uncapped-only", action="store_true",
                    help="time the unswapped runs only (for a per-kernel profile of the plain step)")
    ap.add_argument("--recompute", action="store_true",
                    help="run cheap operations (pooling, concatenation) again late instead of swapping their outputs")
    args = ap.parse_args()
    assert torch.cuda.is_available(), "needs a GPU"
    cap = int(args.cap_gb * GB)
    flags = 0 if args.plain_copies else A.X_ENCODE_SWAPS
    if args.which.startswith("sweep"):
        if args.which == "sweep-resnet":
            spec = W.resnet50(batch=args.batch, size=args.size or 224)
            tensors, label = device_tensors(spec, 8), f"ResNet-50 {args.size or 224}x{args.size or 224}"
        else:
            spec = W.unet3d(batch=args.batch, size=args.size or 192)
            tensors, label = device_tensors(spec, 1), f"3D U-Net {args.size or 192}^3"
        sweep(spec, tensors, label, args.steps, args.warmup, flags)
        return 0
    if args.which == "resnet":
        size = args.size or 224
        b0 = largest_unswapped_batch(cap, size)
        bmax = largest_swapped_batch(cap, size, b0)
        print(json.dumps({"workload": f"ResNet-50 {size}x{size}", "cap_gb": args.cap_gb, "largest_unswapped_batch": b0,
                          "largest_swapped_batch": bmax, "ratio": bmax / b0}), flush=True)
        mult = [float(v) for v in args.multipliers.split(",") if b0 * float(v) < bmax]
        if not args.uncapped_only:
            mult.append(bmax / b0)
        for m in mult:
            batch = int(round(b0 * m))
            spec = W.resnet50(batch=batch, size=size)
            tensors = device_tensors(spec, 8)
            r = run_pair(spec, tensors, cap, args.steps, args.warmup, f"ResNet-50 {size}x{size}", flags, int(args.recompute),
                         args.uncapped_only)
            r["multiple_of_unswapped_batch"] = m
            print(json.dumps(r), flush=True)
            del tensors
            release_memory()
    else:
        size = args.size or 128
        spec = W.unet3d(batch=args.batch, size=size)
        tensors = device_tensors(spec, 1)
        label = f"3D U-Net {size}^3"
        first = run_pair(spec, tensors, cap, args.steps, args.warmup, label, flags)
        print(json.dumps(first), flush=True)
        fp = int(first["unswapped_footprint_gb"] * GB)
        for frac in (float(v) for v in args.fractions.split(",") if not args.uncapped_only):
            r = run_pair(spec, tensors, int(fp * frac), args.steps, args.warmup, label, flags, int(args.recompute))
            r["budget_fraction_of_footprint"] = frac
            print(json.dumps(r), flush=True)


if __name__ == "__main__":
    sys.exit(main())
