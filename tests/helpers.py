"""Shared helpers of the tests: export of a library graph into the oracle's graph structure."""
from oracle.graph import Graph as OGraph, Node as ONode, Edge as OEdge, READ, CONTROL, UPDATE, FWD, BWD, UPD, SWAP

PHASES = {0: FWD, 1: BWD, 2: UPD, 3: SWAP}
KINDS = {0: "param", 1: "input", 2: "target", 3: "const"}
ACTIONS = {0: READ, 1: UPDATE, 2: CONTROL}
SWAP_OUT, SWAP_IN = 21, 22


def to_oracle_graph(g):
    """Structure of a library graph (vertices with phase / variable flag / op code, edges with
    actions) as an oracle Graph; returns (graph, infos)."""
    og = OGraph()
    infos = []
    for i in range(g.node_count()):
        info = g.node_info(i)
        infos.append(info)
        opname = {SWAP_OUT: "swap_out", SWAP_IN: "swap_in"}.get(info.op, f"op{info.op}")
        n = ONode(i, info.name.decode(), "variable" if info.is_variable else opname, {}, bool(info.is_variable),
                  KINDS[info.var_kind] if info.is_variable else None, PHASES[info.phase])
        n.placement = "host" if info.placement == 1 else "device"
        inserted = info.op in (SWAP_OUT, SWAP_IN) or b"/recompute@" in info.name
        n.label = info.gamma if inserted else None
        og.nodes.append(n)
    for e in g.edges():
        og.edges.append(OEdge(e.src, e.dst, ACTIONS[e.action], e.slot))
    return og, infos
