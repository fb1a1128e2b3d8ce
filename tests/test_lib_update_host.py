"""Host-side checks of the update phase: the graph gains one gradient-descent operation and one update edge per
learnable parameter, and variables keep order 0."""
import workloads as W


def test_update_operations_and_edges_are_in_the_graph():
    import paper_1807_02037_amd as L
    A = L.abi
    spec = W.tiny_chain()
    g, ids = L.build_graph(spec, lr=0.1)
    infos = [g.node_info(i) for i in range(g.node_count())]
    ups = [i for i in infos if i.op == A.OP_SGD]
    params = [i for i in infos if i.is_variable and i.var_kind == A.VAR_PARAM]
    assert len(ups) == len(params) > 0 and all(u.phase == A.UPD for u in ups)
    edges = g.edges()
    upd = {(e.src, e.dst) for e in edges if e.action == A.UPDATE}
    assert upd == {(u.id, ids[u.name.decode()[len("update/"):]]) for u in ups}
    # variables keep order 0 although update edges point at them (Definition 2)
    gamma = g.topo_order()
    assert all(gamma[p.id] == 0 for p in params)
