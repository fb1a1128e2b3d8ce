"""Turns a plain-data workload description (a list of layers) into calls of the graph-building ABI."""
from . import _lib as A
from .api import Graph


def build_graph(spec, backward=True, dtype=A.BF16, lr=None, momentum=0.0):
    """Returns (Graph, {name: node id}) with the forward layers of `spec` and, if asked, its backward phase.
    dtype: storage type of the input batch, filters and regression target; A.F32 builds the fp32 check-mode graph
    (every activation then is fp32 and the executor runs its plain fp32 kernels).  lr: if given, the update phase
    (one gradient-descent operation per learnable parameter, with classical momentum if momentum > 0) is appended.  Parameter gradients ("grad/...") and
    updates are declared external: the caller binds memory for them, the memory plan reserves none."""
    g = Graph()
    ids = {}
    xname, xshape = spec["input"]
    ids[xname] = g.add_variable(xname, dtype, xshape, A.VAR_INPUT)
    shape = {xname: tuple(xshape)}
    nd = spec["ndim"]
    for L in spec["layers"]:
        nm = L["name"]
        if L["op"] == "conv":
            cin = shape[L["in"]][-1]
            w = g.add_variable(nm + ".w", dtype, tuple(L["filt"]) + (cin, L["cout"]), A.VAR_PARAM)
            ids[nm + ".w"] = w
            ins, flags = [ids[L["in"]], w], 0
            if L["affine"]:
                for suf in (".scale", ".shift"):
                    ids[nm + suf] = g.add_variable(nm + suf, A.F32, (L["cout"],), A.VAR_PARAM)
                    ins.append(ids[nm + suf])
                flags |= A.F_AFFINE
            if L["bias"]:
                ids[nm + ".b"] = g.add_variable(nm + ".b", A.F32, (L["cout"],), A.VAR_PARAM)
                ins.append(ids[nm + ".b"])
                flags |= A.F_BIAS
            if L["res"] is not None:
                ins.append(ids[L["res"]])
                flags |= A.F_RES
            if L["relu"]:
                flags |= A.F_RELU
            ids[nm] = g.add_op(nm, A.OP_CONV, ins, stride=L["stride"], pad=L["pad"], flags=flags)
        elif L["op"] == "maxpool":
            ids[nm] = g.add_op(nm, A.OP_MAXPOOL, [ids[L["in"]]], filt=(L["win"],) * nd, stride=L["stride"], pad=L["pad"])
        elif L["op"] == "gap":
            ids[nm] = g.add_op(nm, A.OP_GAP, [ids[L["in"]]])
        elif L["op"] == "tconv":
            cin = shape[L["in"]][-1]
            w = g.add_variable(nm + ".w", dtype, (2,) * nd + (cin, L["cout"]), A.VAR_PARAM)
            ids[nm + ".w"] = w
            ids[nm] = g.add_op(nm, A.OP_TCONV, [ids[L["in"]], w])
        elif L["op"] == "concat":
            ids[nm] = g.add_op(nm, A.OP_CONCAT, [ids[s] for s in L["in"]])
        else:
            raise ValueError(L["op"])
        info = g.node_info(ids[nm])
        shape[nm] = tuple(info.dims[i] for i in range(info.ndim))
    loss = spec["loss"]
    oshape = shape[loss["in"]]
    if loss["op"] == "mse":
        t = g.add_variable(loss["target"], dtype, oshape, A.VAR_TARGET)
        ids["loss"] = g.add_op("loss", A.OP_MSE, [ids[loss["in"]], t])
    else:
        t = g.add_variable(loss["target"], A.I32, oshape[:-1], A.VAR_TARGET)
        ids["loss"] = g.add_op("loss", A.OP_SOFTMAX_CE, [ids[loss["in"]], t])
    ids[loss["target"]] = t
    if backward:
        g.build_backward(ids["loss"])
        if lr is not None:
            g.build_update(lr, momentum)
        for i in range(g.node_count()):
            info = g.node_info(i)
            name = info.name.decode()
            if name.startswith("grad/") or name.startswith("update/"):
                ids[name] = i
                # parameter gradients and updated parameters are bound to caller memory by the session
                g.set_external(i)
    return g, ids
