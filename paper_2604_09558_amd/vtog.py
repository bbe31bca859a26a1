"""Which tensors to make virtual: the virtual tensor opportunity graph (Sec. 5.1, Def. 6,
Alg. 1) and the global greedy construction of a points-to graph (Sec. 5.2, Alg. 2).

The two algorithms run inside the library (vt_vtog_build, vt_vtog_greedy, ... of include/vt.h);
this module turns a graph written with tensor names into tensor numbers and back.  A computation
graph is a list of statements ``(out, op, inputs, params)`` (the form the workloads use; ``out``
is a tuple for operators with several outputs) plus the names of the graph's input and output
tensors.  Operators whose kind is not a data-movement operator are compute operators: they
create no opportunities.

An *opportunity* (one edge bundle of the VTOG) says: tensor ``a`` can be made a virtual tensor
of the tensors ``targets`` by eliminating exactly one data-movement operator, in the read
direction (``a`` is an output of the operator; its consumer reads through the map) or in the
store direction (``a`` is an input that lives inside the operator's output; its producer writes
through the map).  Bundles of one tensor exclude each other: that is the conflict set.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass, field

from . import binding

KINDS = dict(binding.OP_KINDS, scatter_nd=binding.OP_SCATTER_ND)


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
    handle: object = None                            # vt_vtog* of the library
    index: dict = field(default_factory=dict)        # tensor name -> number

    @property
    def edges(self):
        return [e for o in self.opportunities for e in o.edges]

    def __del__(self):
        try:
            if self.handle:
                binding.lib().vt_vtog_free(self.handle)
                self.handle = None
        except Exception:
            pass

    def strategy_array(self, chosen):
        """dict tensor -> Opportunity as the library's array (bundle number per tensor, -1 = physical);
        None if some choice is not a bundle of this graph."""
        arr = (C.c_int * len(self.nodes))(*([-1] * len(self.nodes)))
        for t, o in chosen.items():
            if t not in self.index or o not in self.opportunities or o.tensor != t:
                return None
            arr[self.index[t]] = self.opportunities.index(o)
        return arr


def outputs_of(stmt):
    out = stmt[0]
    return tuple(out) if isinstance(out, (tuple, list)) else (out,)


def build_vtog(statements, graph_inputs, graph_outputs, directions=("read", "store")):
    """Alg. 1.  Tensors that are inputs or outputs of the graph stay physical: they get no
    outgoing edge."""
    nodes = list(graph_inputs)
    for st in statements:
        for o in outputs_of(st):
            if o not in nodes:
                nodes.append(o)
    for st in statements:                     # names that only ever appear as inputs (index tensors and the like)
        for i in st[2]:
            if isinstance(i, str) and i not in nodes:
                nodes.append(i)
    index = {n: k for k, n in enumerate(nodes)}
    arr = (binding.VtGraphStmt * max(1, len(statements)))()
    for k, st in enumerate(statements):
        ins = [i for i in st[2] if isinstance(i, str)]
        outs = outputs_of(st)
        kind = KINDS.get(st[1], binding.OP_COMPUTE)
        if st[1] == "split" and len(outs) < len(st[3].get("sizes", outs)):
            # a statement that names one output of a Split (the executable chains' form) is a Slice as
            # far as the graph goes: its input cannot be stitched from outputs that are not all there,
            # so it gets the read-direction bundle only
            kind = KINDS["slice"]
        arr[k].kind = kind
        arr[k].n_in, arr[k].n_out = len(ins), len(outs)
        for j, i in enumerate(ins):
            arr[k].in_[j] = index[i]
        for j, o in enumerate(outs):
            arr[k].out[j] = index[o]
    pinned = (C.c_uint8 * len(nodes))(*[1 if n in set(graph_inputs) | set(graph_outputs) else 0 for n in nodes])
    mask = (binding.DIR_READ if "read" in directions else 0) | (binding.DIR_STORE if "store" in directions else 0)
    h = C.c_void_p()
    L = binding.lib()
    binding._check(L.vt_vtog_build(arr, len(statements), len(nodes), pinned, mask, C.byref(h)))
    g = Vtog(nodes, [], handle=h, index=index)
    nb = C.c_int()
    binding._check(L.vt_vtog_size(h, None, C.byref(nb)))
    for b in range(nb.value):
        t, nt, st, dr = C.c_int(), C.c_int(), C.c_int(), C.c_int()
        tg = (C.c_int * binding.VT_MAX_OP_INPUTS)()
        binding._check(L.vt_vtog_bundle(h, b, C.byref(t), C.byref(nt), tg, C.byref(st), C.byref(dr)))
        opp = Opportunity(nodes[t.value], tuple(nodes[tg[i]] for i in range(nt.value)), st.value,
                          "read" if dr.value == binding.DIR_READ else "store")
        g.opportunities.append(opp)
        g.by_tensor.setdefault(opp.tensor, []).append(opp)
    return g


def is_points_to_graph(vtog, chosen):
    """`chosen`: tensor -> Opportunity.  Valid if every choice is one of the tensor's bundles
    (at most one each, so no two conflict) and following the edges always ends at a physical
    tensor (no cycle)."""
    arr = vtog.strategy_array(chosen)
    if arr is None:
        return False
    ok = C.c_int()
    binding._check(binding.lib().vt_vtog_is_points_to_graph(vtog.handle, arr, C.byref(ok)))
    return bool(ok.value)


def greedy(vtog, profile):
    """Alg. 2 (runs in the library).  ``profile(opportunity, chosen)`` returns the latency saving of
    adding that bundle to the strategy ``chosen`` (dict tensor -> Opportunity), i.e. the sum of w(e)
    over its edges.  Returns (chosen, total saving, [(opportunity, its saving) in the order taken])."""
    n = len(vtog.nodes)
    seen = {}

    failure = []

    def saving(_user, b, arr):
        if failure:                      # an exception cannot cross the library: stop the search, raise afterwards
            return -1.0
        try:
            chosen = {vtog.nodes[t]: vtog.opportunities[arr[t]] for t in range(n) if arr[t] >= 0}
            w = float(profile(vtog.opportunities[b], chosen))
        except BaseException as e:       # noqa: B902
            failure.append(e)
            return -1.0
        seen[b] = w
        return w

    out = (C.c_int * n)()
    order = (C.c_int * n)()
    total, n_order = C.c_double(), C.c_int()
    cb = binding.SAVING_FN(saving)
    binding._check(binding.lib().vt_vtog_greedy(vtog.handle, cb, None, out, C.byref(total), order, C.byref(n_order)))
    if failure:
        raise failure[0]
    chosen = {vtog.nodes[t]: vtog.opportunities[out[t]] for t in range(n) if out[t] >= 0}
    trace = [(vtog.opportunities[order[k]], seen[order[k]]) for k in range(n_order.value)]
    return chosen, total.value, trace


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
