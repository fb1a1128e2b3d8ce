"""Plain-data descriptions of the synthetic workloads and their seeded tensors.

A workload is a dict
    {"name", "ndim" (2 or 3 spatial dims), "input": (name, shape), "layers": [...], "loss": {...}}
with channels-last shapes (N, H, W, C) or (N, D, H, W, C).  Each layer is a dict
with "name", "op" and "in"; see the builders below for the fields of each op.
Both the oracle and the GPU library build their own graphs from these lists.

The workloads stand in for the models the paper measures (ResNet-50 at 224x224
and a 3DUnet at 128^3 / 192^3, Section 6): only shapes and class counts are
taken from there, all values are seeded synthetic draws.
"""
import math
import numpy as np

from . import rng

BASE_SEED = 1807020370


def _conv(name, src, filt, cout, stride=1, pad=0, relu=True, res=None, affine=False, bias=False):
    return {"name": name, "op": "conv", "in": src, "filt": tuple(filt), "cout": cout, "stride": stride,
            "pad": pad, "relu": relu, "res": res, "affine": affine, "bias": bias}


def tiny_chain(batch=2, size=32, cin=3, width=16, depth=4, classes=10):
    """Config 1: conv3x3+ReLU chain, global average pool, linear, MSE."""
    layers, src = [], "x"
    for i in range(depth):
        layers.append(_conv(f"conv{i + 1}", src, (3, 3), width, 1, 1, relu=True))
        src = f"conv{i + 1}"
    layers.append({"name": "gap", "op": "gap", "in": src})
    layers.append(_conv("fc", "gap", (1, 1), classes, relu=False, bias=True))
    return {"name": "tiny_chain", "cfg": 1, "ndim": 2, "input": ("x", (batch, size, size, cin)),
            "layers": layers, "loss": {"op": "mse", "in": "fc", "target": "t"}}


def bottleneck_stage(batch=64, size=56, cin=256, width=64, blocks=3):
    """Config 2: ResNet-50 conv2_x stage, identity shortcuts, no normalisation, MSE on the output."""
    layers, src = [], "x"
    for b in range(blocks):
        p = f"b{b + 1}"
        layers.append(_conv(p + "a", src, (1, 1), width, relu=True))
        layers.append(_conv(p + "b", p + "a", (3, 3), width, 1, 1, relu=True))
        layers.append(_conv(p + "c", p + "b", (1, 1), cin, relu=True, res=src))
        src = p + "c"
    return {"name": "bottleneck_stage", "cfg": 2, "ndim": 2, "input": ("x", (batch, size, size, cin)),
            "layers": layers, "loss": {"op": "mse", "in": src, "target": "t"}}


def resnet50(batch=2, size=224, classes=1000, stage_blocks=(3, 4, 6, 3), base=64):
    """Config 3: ResNet-50 topology with a per-channel affine in place of batch norm.

    Stride sits on the first 1x1 of a stage's first block (the original layout
    of the network the paper cites)."""
    layers = [_conv("stem", "x", (7, 7), base, 2, 3, relu=True, affine=True),
              {"name": "pool", "op": "maxpool", "in": "stem", "win": 3, "stride": 2, "pad": 1}]
    src = "pool"
    for s, nb in enumerate(stage_blocks):
        width = base * (2 ** s)
        out = 4 * width
        for b in range(nb):
            p = f"s{s + 2}b{b + 1}"
            stride = 2 if (b == 0 and s > 0) else 1
            if b == 0:
                layers.append(_conv(p + "p", src, (1, 1), out, stride, 0, relu=False, affine=True))
                short = p + "p"
            else:
                short = src
            layers.append(_conv(p + "a", src, (1, 1), width, stride, 0, relu=True, affine=True))
            layers.append(_conv(p + "b", p + "a", (3, 3), width, 1, 1, relu=True, affine=True))
            layers.append(_conv(p + "c", p + "b", (1, 1), out, 1, 0, relu=True, res=short, affine=True))
            src = p + "c"
    layers.append({"name": "gap", "op": "gap", "in": src})
    layers.append(_conv("fc", "gap", (1, 1), classes, relu=False, bias=True))
    return {"name": "resnet50", "cfg": 3, "ndim": 2, "input": ("x", (batch, size, size, 3)),
            "layers": layers, "loss": {"op": "softmax_ce", "in": "fc", "target": "t", "classes": classes}}


def unet3d(batch=1, size=128, base=32, levels=4, classes=4, cin=1):
    """Configs 4/5: 3D U-Net style encoder-decoder (levels-1 poolings and up-convolutions)."""
    layers, src, skips = [], "x", []
    for l in range(levels):
        w = base * (2 ** l)
        layers.append(_conv(f"e{l}a", src, (3, 3, 3), w, 1, 1, relu=True))
        layers.append(_conv(f"e{l}b", f"e{l}a", (3, 3, 3), w, 1, 1, relu=True))
        src = f"e{l}b"
        if l < levels - 1:
            skips.append(src)
            layers.append({"name": f"p{l}", "op": "maxpool", "in": src, "win": 2, "stride": 2, "pad": 0})
            src = f"p{l}"
    for l in range(levels - 2, -1, -1):
        w = base * (2 ** l)
        layers.append({"name": f"u{l}", "op": "tconv", "in": src, "cout": w})
        layers.append({"name": f"cat{l}", "op": "concat", "in": [skips[l], f"u{l}"]})
        layers.append(_conv(f"d{l}a", f"cat{l}", (3, 3, 3), w, 1, 1, relu=True))
        layers.append(_conv(f"d{l}b", f"d{l}a", (3, 3, 3), w, 1, 1, relu=True))
        src = f"d{l}b"
    layers.append(_conv("head", src, (1, 1, 1), classes, relu=False))
    return {"name": "unet3d", "cfg": 4, "ndim": 3, "input": ("x", (batch, size, size, size, cin)),
            "layers": layers, "loss": {"op": "softmax_ce", "in": "head", "target": "t", "classes": classes}}


def pool_net(batch=2, size=12, cin=8, width=16):
    """Small 2-D net exercising overlapping max pooling, strides, a projection shortcut and affine."""
    layers = [_conv("c1", "x", (3, 3), width, 1, 1, relu=True, affine=True),
              {"name": "pool", "op": "maxpool", "in": "c1", "win": 3, "stride": 2, "pad": 1},
              _conv("c2p", "pool", (1, 1), 2 * width, 2, 0, relu=False, affine=True),
              _conv("c2a", "pool", (3, 3), width, 2, 1, relu=True, affine=True),
              _conv("c2b", "c2a", (1, 1), 2 * width, 1, 0, relu=True, res="c2p", affine=True),
              {"name": "gap", "op": "gap", "in": "c2b"},
              _conv("fc", "gap", (1, 1), 12, relu=False, bias=True)]
    return {"name": "pool_net", "cfg": 6, "ndim": 2, "input": ("x", (batch, size, size, cin)),
            "layers": layers, "loss": {"op": "softmax_ce", "in": "fc", "target": "t", "classes": 12}}


def updown_net(batch=1, size=8, cin=8, width=16, ndim=3):
    """Small net (3-D, or 2-D with ndim=2) exercising 2x2(x2) pooling, transposed convolution, concatenation and a
    4-class head."""
    f3, f1 = (3,) * ndim, (1,) * ndim
    layers = [_conv("e0", "x", f3, width, 1, 1, relu=True),
              {"name": "p0", "op": "maxpool", "in": "e0", "win": 2, "stride": 2, "pad": 0},
              _conv("e1", "p0", f3, 2 * width, 1, 1, relu=True),
              {"name": "u0", "op": "tconv", "in": "e1", "cout": width},
              {"name": "cat0", "op": "concat", "in": ["e0", "u0"]},
              _conv("d0", "cat0", f3, width, 1, 1, relu=True),
              _conv("head", "d0", f1, 4, relu=False)]
    return {"name": "updown_net", "cfg": 7, "ndim": ndim, "input": ("x", (batch,) + (size,) * ndim + (cin,)),
            "layers": layers, "loss": {"op": "softmax_ce", "in": "head", "target": "t", "classes": 4}}


def infer_shapes(spec):
    """Shapes of every activation and parameter: {"act": {name: shape}, "param": {name: shape}}."""
    nd = spec["ndim"]
    act = {spec["input"][0]: tuple(spec["input"][1])}
    par = {}
    for L in spec["layers"]:
        op = L["op"]
        if op == "concat":
            a, b = (act[s] for s in L["in"])
            assert a[:-1] == b[:-1], (L["name"], a, b)
            act[L["name"]] = a[:-1] + (a[-1] + b[-1],)
            continue
        s = act[L["in"]]
        n, sp, c = s[0], s[1:-1], s[-1]
        if op == "conv":
            f = L["filt"]
            osp = tuple((sp[i] + 2 * L["pad"] - f[i]) // L["stride"] + 1 for i in range(nd))
            act[L["name"]] = (n,) + osp + (L["cout"],)
            par[L["name"] + ".w"] = tuple(f) + (c, L["cout"])
            if L["affine"]:
                par[L["name"] + ".scale"] = (L["cout"],)
                par[L["name"] + ".shift"] = (L["cout"],)
            if L["bias"]:
                par[L["name"] + ".b"] = (L["cout"],)
            if L["res"] is not None:
                assert act[L["res"]] == act[L["name"]], (L["name"], act[L["res"]], act[L["name"]])
        elif op == "maxpool":
            osp = tuple((sp[i] + 2 * L["pad"] - L["win"]) // L["stride"] + 1 for i in range(nd))
            act[L["name"]] = (n,) + osp + (c,)
        elif op == "gap":
            act[L["name"]] = (n,) + (1,) * nd + (c,)
        elif op == "tconv":
            act[L["name"]] = (n,) + tuple(2 * d for d in sp) + (L["cout"],)
            par[L["name"] + ".w"] = (2,) * nd + (c, L["cout"])
        else:
            raise ValueError(op)
    return {"act": act, "param": par}


def tensor_seed(cfg, index):
    return BASE_SEED + 1000 * cfg + index


def make_tensors(spec, affine="unit", seed_cfg=None):
    """Seeded host tensors of a workload, as fp64 arrays.

    Input, convolution weights and an MSE target are N(0,1) / He-normal draws
    rounded once to bfloat16 (so storage in bf16 loses nothing); labels are
    int32.  Affine scale/shift and biases are fp32-representable: with
    affine="unit" they are 1 / 0 / 0 (the configured initialisation), with
    affine="random" they are small seeded perturbations around those values so
    that tests exercise the affine and bias terms.
    """
    shp = infer_shapes(spec)
    cfg = spec["cfg"] if seed_cfg is None else seed_cfg
    out, idx = {}, 0
    xname, xshape = spec["input"]
    out[xname] = rng.round_to_bf16(rng.normal(tensor_seed(cfg, idx), xshape))
    idx += 1
    for L in spec["layers"]:
        for suffix in (".w", ".scale", ".shift", ".b"):
            pname = L["name"] + suffix
            if pname not in shp["param"]:
                continue
            ps = shp["param"][pname]
            if suffix == ".w":
                fan_in = int(np.prod(ps[:-1]))
                v = rng.round_to_bf16(rng.normal(tensor_seed(cfg, idx), ps, math.sqrt(2.0 / fan_in)))
            else:
                base = 1.0 if suffix == ".scale" else 0.0
                if suffix == ".scale" and spec["name"] == "resnet50" and (L["res"] is not None or L["name"].endswith("p")):
                    # last affine of a residual branch and of a projection shortcut: keeps activations O(1)
                    # through 16 blocks, as the normalisation it replaces would
                    base = 0.25 if L["res"] is not None else 0.5
                if affine == "random":
                    v = base + rng.normal(tensor_seed(cfg, idx), ps, 0.1)
                else:
                    v = np.full(ps, base)
                v = v.astype(np.float32).astype(np.float64)
            out[pname] = v
            idx += 1
    loss = spec["loss"]
    oshape = shp["act"][loss["in"]]
    if loss["op"] == "mse":
        out[loss["target"]] = rng.round_to_bf16(rng.normal(tensor_seed(cfg, 900), oshape))
    else:
        out[loss["target"]] = rng.uniform_int(tensor_seed(cfg, 900), oshape[:-1], loss["classes"])
    return out
