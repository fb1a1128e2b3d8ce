"""Variants of the oracle's bf16 storage marks ("q" attributes of oracle/model.py), for tests that ask how much
the placement of the roundings matters.  Test helper; holds none of the layer arithmetic."""
from oracle import evaluate, model
from oracle.graph import BWD


def run_with_marks(spec, tensors, marks):
    """One oracle step with a chosen set of rounding marks.  marks: "model" (as oracle/model.py sets them),
    "none", "all_backward" (the model's forward marks, and every backward activation gradient rounded, fused into
    a later sum / mask or not), or a set of layer names (only those forward outputs are rounded).
    Returns {name: value} like evaluate.train_step."""
    g, ids = model.build(spec)
    if marks == "none":
        val = evaluate.run(g, tensors, False)
    else:
        if marks == "all_backward":
            for n in g.nodes:
                if not n.is_var and n.phase == BWD and not n.name.startswith("grad/"):
                    n.attrs["q"] = True
        elif marks != "model":
            chosen = {ids[name] for name in marks}
            for n in g.nodes:
                if not n.is_var:
                    n.attrs["q"] = n.id in chosen
        val = evaluate.run(g, tensors, True)
    return {name: val[v] for name, v in ids.items() if not g.nodes[v].is_var}
