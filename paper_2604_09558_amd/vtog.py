"""Which tensors to make virtual: the virtual tensor opportunity graph (Sec. 5.1, Def. 6,
Alg. 1) and the global greedy construction of a points-to graph (Sec. 5.2, Alg. 2).

Host logic only.  A computation graph is a list of statements ``(out, op, inputs, params)`` (the
form the workloads use; ``out`` is a tuple for operators with several outputs) plus the names of
the graph's input and output tensors.  Operators whose kind is not a data-movement operator are
compute operators: they create no opportunities.

An *opportunity* (one edge bundle of the VTOG) says: tensor ``a`` can be made a virtual tensor
of the tensors ``targets`` by eliminating exactly one data-movement operator.  Two directions:

  read   ``a`` is an output of the operator and its elements are found in the operator's inputs
         (the consumer of ``a`` reads through the map);
  store  ``a`` is an input of the operator and lives inside the operator's output (the producer
         of ``a`` writes through the map): inputs of Concat, the input of a Reshape or Permute,
         the updates and the data input of a ScatterND.

Rules per operator follow Sec. 4.4.  All edges of a bundle are taken together (the output of a
Concat is a virtual tensor of all of its inputs at once); bundles of one tensor that come from
different operators, or from different directions of one operator, are mutually exclusive (a
tensor mapped into two places would break the one-to-one property): that is the conflict set.
"""
from __future__ import annotations

from dataclasses import dataclass, field

READ_OPS = ("reshape", "permute", "slice", "unsqueeze", "expand", "index_select", "split", "concat", "scatter_nd")
BIJECTIVE = ("reshape", "permute", "unsqueeze")


@dataclass(frozen=True)
class Opportunity:
    tensor: str            # the tensor that becomes virtual
    targets: tuple         # the tensors it points to (one edge of the VTOG each)
    op_index: int          # the statement that is eliminated
    direction: str         # "read" or "store"

    @property
    def edges(self):
        return tuple((self.tensor, t) for t in self.targets)


@dataclass
class Vtog:
    nodes: list
    opportunities: list                              # every bundle, in statement order
    by_tensor: dict = field(default_factory=dict)    # tensor -> its bundles (the conflict set: pick at most one)

    @property
    def edges(self):
        return [e for o in self.opportunities for e in o.edges]


def outputs_of(stmt):
    out = stmt[0]
    return tuple(out) if isinstance(out, (tuple, list)) else (out,)


def vt_rules(stmt, index):
    """Opportunities one data-movement statement creates (Sec. 4.4), both directions."""
    _, op, ins, _ = stmt
    outs = outputs_of(stmt)
    res = []
    if op not in READ_OPS:
        return res
    if op == "scatter_nd":
        data, _, updates = ins[0], ins[1], ins[2]
        # the output starts as a clone of `data`: output as a virtual tensor of data (Type I),
        # and `updates` as a virtual tensor of the output (Type II: the indices may scatter)
        res.append(Opportunity(outs[0], (data,), index, "read"))
        res.append(Opportunity(updates, (outs[0],), index, "store"))
        return res
    if op == "split":
        for o in outs:
            res.append(Opportunity(o, (ins[0],), index, "read"))
        res.append(Opportunity(ins[0], outs, index, "store"))        # the input stitched from its outputs: Type II
        return res
    if op == "concat":
        res.append(Opportunity(outs[0], tuple(ins), index, "read"))
        for i in ins:
            res.append(Opportunity(i, (outs[0],), index, "store"))
        return res
    res.append(Opportunity(outs[0], (ins[0],), index, "read"))
    if op in BIJECTIVE:
        res.append(Opportunity(ins[0], (outs[0],), index, "store"))
    return res


def build_vtog(statements, graph_inputs, graph_outputs, directions=("read", "store")):
    """Alg. 1.  Tensors that are inputs or outputs of the graph stay physical: they get no
    outgoing edge."""
    nodes = list(graph_inputs)
    for st in statements:
        for o in outputs_of(st):
            if o not in nodes:
                nodes.append(o)
    pinned = set(graph_inputs) | set(graph_outputs)
    g = Vtog(nodes, [])
    for k, st in enumerate(statements):
        for opp in vt_rules(st, k):
            if opp.direction in directions and opp.tensor not in pinned:
                g.opportunities.append(opp)
                g.by_tensor.setdefault(opp.tensor, []).append(opp)
    return g


def is_points_to_graph(vtog, chosen):
    """`chosen`: tensor -> Opportunity.  Valid if every choice is one of the tensor's bundles
    (at most one each, so no two conflict) and following the edges always ends at a physical
    tensor (no cycle)."""
    for t, o in chosen.items():
        if o not in vtog.by_tensor.get(t, []):
            return False
    state = {}

    def grounded(t):
        if t not in chosen:
            return True
        if state.get(t) == 1:
            return False
        if state.get(t) == 2:
            return True
        state[t] = 1
        ok = all(grounded(x) for x in chosen[t].targets)
        state[t] = 2
        return ok

    return all(grounded(t) for t in chosen)


def greedy(vtog, profile):
    """Alg. 2.  ``profile(opportunity, chosen)`` returns the latency saving of adding that bundle
    to the strategy ``chosen`` (dict tensor -> Opportunity), i.e. the sum of w(e) over its edges.

    Reading of the listing where it leaves room: MaxEdges(v, S(v), A) ranges over the bundles of v
    whose targets all lie in the anchor set A (bundles of one tensor exclude each other, so the
    best non-conflicting edge set is the best single bundle); a tensor without such a bundle is
    not a candidate in that iteration; when the best candidate saves nothing (< 0) the loop stops
    and every tensor left over stays physical.  After a tensor joins, the bundles that point to it
    are profiled again against the grown strategy."""
    anchors = {v for v in vtog.nodes if not vtog.by_tensor.get(v)}
    chosen = {}
    w = {o: profile(o, dict(chosen)) for o in vtog.opportunities}
    total = 0.0
    trace = []
    while len(anchors) < len(vtog.nodes):
        best = None
        for v in vtog.nodes:
            if v in anchors:
                continue
            for o in vtog.by_tensor[v]:
                if all(t in anchors for t in o.targets) and (best is None or w[o] > w[best]):
                    best = o
        if best is None or w[best] < 0:
            break
        anchors.add(best.tensor)
        chosen[best.tensor] = best
        total += w[best]
        trace.append((best, w[best]))
        for o in vtog.opportunities:
            if best.tensor in o.targets and o.tensor not in anchors:
                w[o] = profile(o, dict(chosen))
    return chosen, total, trace


def read_chain(statements, chosen, tensor):
    """Statements that must be composed into the descriptor of `tensor`, and the physical
    tensors the descriptor reads, for a strategy of read-direction choices."""
    by_out = {}
    for k, st in enumerate(statements):
        for o in outputs_of(st):
            by_out[o] = k
    keep, sources, seen = set(), [], set()

    def walk(t):
        if t in seen:
            return
        seen.add(t)
        o = chosen.get(t)
        if o is None or o.direction != "read":
            if t not in sources:
                sources.append(t)
            return
        keep.add(by_out[t])
        for x in statements[by_out[t]][2]:
            if isinstance(x, str):
                walk(x)

    walk(tensor)
    return [statements[k] for k in sorted(keep)], sources
