"""Computational graph G = (V, E, lambda, tau) and its topological ordering.

TEST INFRASTRUCTURE ONLY; nothing in the product path may import it.

Follows Section 3 (Definition 1, Table 1 "Notations", Definition 2):
vertices are operations, each tagged normal or parameterised (variables and
constants are parameterised); edges carry a tensor and one of the actions
read / update / control.
"""

READ, UPDATE, CONTROL = "read", "update", "control"
FWD, BWD, UPD, SWAP = "fwd", "bwd", "upd", "swap"


class Node:
    __slots__ = ("id", "name", "op", "attrs", "is_var", "kind", "phase", "placement", "label")

    def __init__(self, id, name, op, attrs, is_var, kind, phase):
        self.id, self.name, self.op, self.attrs = id, name, op, dict(attrs or {})
        self.is_var, self.kind, self.phase = is_var, kind, phase
        self.placement = "device"
        self.label = None          # order the rewriter assigns to an inserted vertex (Figure 3)

    def __repr__(self):
        return f"<{self.id}:{self.name}:{self.op}:{self.phase}>"


class Edge:
    __slots__ = ("src", "dst", "action", "slot")

    def __init__(self, src, dst, action, slot=-1):
        self.src, self.dst, self.action, self.slot = src, dst, action, slot

    def key(self):
        return (self.src, self.dst, self.action, self.slot)


class Graph:
    def __init__(self):
        self.nodes = []
        self.edges = []

    # ---- construction -------------------------------------------------
    def add_variable(self, name, kind="param", attrs=None):
        n = Node(len(self.nodes), name, "variable", attrs, True, kind, FWD)
        self.nodes.append(n)
        return n.id

    def add_op(self, name, op, inputs, phase=FWD, attrs=None):
        n = Node(len(self.nodes), name, op, attrs, False, None, phase)
        self.nodes.append(n)
        for slot, src in enumerate(inputs):
            self.edges.append(Edge(src, n.id, READ, slot))
        return n.id

    def add_update_edge(self, src, var):
        assert self.nodes[var].is_var
        self.edges.append(Edge(src, var, UPDATE))

    def add_control_edge(self, src, dst):
        # Section 3.2: there is no control edge into a variable
        assert not self.nodes[dst].is_var
        self.edges.append(Edge(src, dst, CONTROL))

    def copy(self):
        g = Graph()
        for n in self.nodes:
            m = Node(n.id, n.name, n.op, n.attrs, n.is_var, n.kind, n.phase)
            m.placement, m.label = n.placement, n.label
            g.nodes.append(m)
        g.edges = [Edge(e.src, e.dst, e.action, e.slot) for e in self.edges]
        return g

    # ---- queries --------------------------------------------------------
    def inputs(self, v):
        """Data inputs of v in slot order."""
        es = sorted((e for e in self.edges if e.dst == v and e.action == READ), key=lambda e: e.slot)
        return [e.src for e in es]

    def control_inputs(self, v):
        return [e.src for e in self.edges if e.dst == v and e.action == CONTROL]

    def out(self, u):
        """Out(u): operations with a read or control edge from u (update edges lead to variables)."""
        return sorted({e.dst for e in self.edges if e.src == u and e.action != UPDATE})

    def readers(self, u):
        return sorted({e.dst for e in self.edges if e.src == u and e.action == READ})

    def gamma(self):
        """Topological ordering of Definition 2, taken as minimal levels: 0 for every
        parameterised vertex, otherwise 1 + the largest order among the sources of incoming
        read and control edges.  Update edges end in variables and change no order."""
        preds = {n.id: [] for n in self.nodes}
        succs = {n.id: [] for n in self.nodes}
        for e in self.edges:
            if e.action == UPDATE or self.nodes[e.dst].is_var:
                continue
            preds[e.dst].append(e.src)
            succs[e.src].append(e.dst)
        indeg = {v: len(p) for v, p in preds.items()}
        gam = {}
        ready = [v for v, d in indeg.items() if d == 0]
        done = 0
        while ready:
            v = ready.pop()
            done += 1
            if self.nodes[v].is_var:
                gam[v] = 0
            else:
                gam[v] = 1 + max((gam[p] for p in preds[v]), default=0)
            for s in succs[v]:
                indeg[s] -= 1
                if indeg[s] == 0:
                    ready.append(s)
        if done != len(self.nodes):
            raise ValueError("graph has a cycle")
        return gam

    def reach(self, u):
        """Reach(u): vertices reachable from u along read and control edges (u excluded)."""
        succs = {}
        for e in self.edges:
            if e.action != UPDATE:
                succs.setdefault(e.src, []).append(e.dst)
        seen, stack = set(), [u]
        while stack:
            a = stack.pop()
            for b in succs.get(a, ()):
                if b not in seen:
                    seen.add(b)
                    stack.append(b)
        return seen
