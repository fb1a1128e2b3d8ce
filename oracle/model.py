"""Graph of a workload: one forward pass and its back-propagation (Section 3.3).

TEST INFRASTRUCTURE ONLY; nothing in the product path may import it.

Every layer of a workload description becomes a few unfused vertices
(convolution, affine, bias, add, ReLU ...), and every forward vertex that has
a learnable parameter upstream gets its backward vertices, tagged BWD, which
read the forward tensors they need -- the forward-to-backward edges that the
rewriting of Section 4 acts on.  The input batch and targets are variables
that are not learnable, so no gradient flows into them.
"""
from .graph import Graph, FWD, BWD


def build(spec):
    """Returns (graph, names) where names maps a layer / parameter / "loss" /
    "grad/<param>" name to its vertex id."""
    g = Graph()
    ids = {}
    xname = spec["input"][0]
    ids[xname] = g.add_variable(xname, "input")
    fwd_ops = []          # forward op vertices in creation order
    learn = set()         # vertices with a learnable parameter upstream (themselves included)

    def var(name, kind="param"):
        ids[name] = g.add_variable(name, kind)
        if kind == "param":
            learn.add(ids[name])
        return ids[name]

    def op(name, kind, ins, attrs=None):
        v = g.add_op(name, kind, ins, FWD, attrs)
        fwd_ops.append(v)
        if any(i in learn for i in ins):
            learn.add(v)
        return v

    for L in spec["layers"]:
        nm = L["name"]
        if L["op"] == "conv":
            w = var(nm + ".w")
            chain = [("conv", [ids[L["in"]], w], {"stride": L["stride"], "pad": L["pad"]})]
            if L["affine"]:
                chain.append(("affine", [var(nm + ".scale"), var(nm + ".shift")], None))
            if L["bias"]:
                chain.append(("bias", [var(nm + ".b")], None))
            if L["res"] is not None:
                chain.append(("add", [ids[L["res"]]], None))
            if L["relu"]:
                chain.append(("relu", [], None))
            cur = None
            for i, (kind, ins, attrs) in enumerate(chain):
                last = i == len(chain) - 1
                full = ins if cur is None else [cur] + ins
                a = dict(attrs or {})
                a["q"] = last
                cur = op(nm if last else f"{nm}/{kind}", kind, full, a)
            ids[nm] = cur
        elif L["op"] == "maxpool":
            ids[nm] = op(nm, "maxpool", [ids[L["in"]]],
                         {"win": L["win"], "stride": L["stride"], "pad": L["pad"], "q": True})
        elif L["op"] == "gap":
            ids[nm] = op(nm, "gap", [ids[L["in"]]], {"q": True})
        elif L["op"] == "tconv":
            ids[nm] = op(nm, "tconv", [ids[L["in"]], var(nm + ".w")], {"q": True})
        elif L["op"] == "concat":
            ids[nm] = op(nm, "concat", [ids[s] for s in L["in"]], {"q": True})
        else:
            raise ValueError(L["op"])

    loss = spec["loss"]
    t = var(loss["target"], "target")
    ids["loss"] = op("loss", loss["op"], [ids[loss["in"]], t])

    # ---- back-propagation: walk the forward vertices in reverse ---------------------------
    contrib = {}          # forward vertex -> gradient vertices to be summed

    def bop(name, kind, ins, attrs=None):
        return g.add_op(name, kind, ins, BWD, attrs)

    def give(v, gv):
        if v in learn:
            contrib.setdefault(v, []).append(gv)

    def total(v):
        parts = contrib[v]
        acc = parts[0]
        for i, pgrad in enumerate(parts[1:]):
            acc = bop(f"{g.nodes[v].name}/gsum{i}", "add", [acc, pgrad])
        return acc

    for v in reversed(fwd_ops):
        n = g.nodes[v]
        ins = g.inputs(v)
        if n.op in ("mse", "softmax_ce"):
            give(ins[0], bop("loss/grad", n.op + "_bwd", [ins[0], ins[1]]))
            continue
        if v not in contrib:
            continue
        dy = total(v)
        nm = n.name
        if n.op == "relu":
            give(ins[0], bop(nm + "/relu_grad", "relu_grad", [dy, v]))
        elif n.op == "add":
            give(ins[0], dy)
            give(ins[1], dy)
        elif n.op == "bias":
            give(ins[0], dy)
            ids["grad/" + g.nodes[ins[1]].name] = bop("grad/" + g.nodes[ins[1]].name, "bias_grad", [dy])
        elif n.op == "affine":
            ids["grad/" + g.nodes[ins[1]].name] = bop("grad/" + g.nodes[ins[1]].name, "affine_dscale", [dy, ins[0]])
            ids["grad/" + g.nodes[ins[2]].name] = bop("grad/" + g.nodes[ins[2]].name, "bias_grad", [dy])
            give(ins[0], bop(nm + "/affine_dx", "affine_dx", [dy, ins[1]]))
        elif n.op == "conv":
            a = {"stride": n.attrs["stride"], "pad": n.attrs["pad"], "shape_of": ins[0], "filt_of": ins[1]}
            ids["grad/" + g.nodes[ins[1]].name] = bop("grad/" + g.nodes[ins[1]].name, "conv_wgrad", [ins[0], dy], a)
            if ins[0] in learn:
                give(ins[0], bop(nm + "/dgrad", "conv_dgrad", [dy, ins[1]], a))
        elif n.op == "tconv":
            ids["grad/" + g.nodes[ins[1]].name] = bop("grad/" + g.nodes[ins[1]].name, "tconv_wgrad", [ins[0], dy])
            if ins[0] in learn:
                give(ins[0], bop(nm + "/dgrad", "tconv_dgrad", [dy, ins[1]]))
        elif n.op == "maxpool":
            give(ins[0], bop(nm + "/bwd", "maxpool_bwd", [dy, ins[0]], dict(n.attrs, q=False)))
        elif n.op == "gap":
            give(ins[0], bop(nm + "/bwd", "gap_bwd", [dy], {"shape_of": ins[0]}))
        elif n.op == "concat":
            give(ins[0], bop(nm + "/bwd_a", "slice_c", [dy], {"shape_of": ins[0], "second": False}))
            give(ins[1], bop(nm + "/bwd_b", "slice_c", [dy], {"shape_of": ins[0], "second": True}))
        else:
            raise ValueError(n.op)

    # backward tensors the GPU path stores in bf16: every backward activation gradient
    # except one that only feeds a sum or a ReLU mask (those are applied before storing)
    for n in g.nodes:
        if n.phase != BWD or n.name.startswith("grad/"):
            continue
        cons = [g.nodes[c] for c in g.readers(n.id)]
        fused = bool(cons) and all(
            c.phase == BWD and (c.op == "add" or (c.op == "relu_grad" and g.inputs(c.id)[0] == n.id))
            for c in cons)
        n.attrs["q"] = not fused
    return g, ids
