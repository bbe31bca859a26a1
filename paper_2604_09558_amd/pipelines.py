"""The two ways to run a workload on the GPU, as sequences of library calls.

virtual:       build the descriptors of the consumer's inputs, launch the consumer.  No
               intermediate of the chain exists in memory.
materialized:  execute the chain's data-movement operators as explicit copy kernels into fresh
               dense buffers (every operator, "full"), then launch the SAME consumer on
               identity descriptors of the dense results.  This is the on-GPU comparison path.

Only launches and buffer bookkeeping happen here; all arithmetic is in the library.
"""
from __future__ import annotations

import torch

from . import binding as vt
from .torch_io import TORCH_DTYPE, DeviceWorkload


class Materialized:
    """Runs a chain op by op with vt_copy_op.  Buffers are allocated once (outside any timed
    region) and reused by `run`."""

    def __init__(self, dw: DeviceWorkload, wanted):
        self.dw = dw
        wl = dw.wl
        defs = {out: (op, ins, p) for out, op, ins, p in wl.chain}
        order, seen = [], set()

        def visit(n):
            if n in seen or n not in defs:
                return
            seen.add(n)
            for i in defs[n][1]:
                visit(i)
            order.append(n)

        for w in wanted:
            visit(w)
        self.order = order
        self.defs = defs
        self.shapes = {k: tuple(t.shape) for k, t in dw.tensors.items()}
        self.bufs = dict(dw.tensors)
        self.bytes_written = 0
        for n in order:
            op, ins, p = defs[n]
            d = vt.build_chain([(n, op, ins, p)], {i: (self.shapes[i], wl.dtype) for i in ins}, n, wl.index_tables)
            self.shapes[n] = d.shape
            self.bufs[n] = torch.empty(d.shape, dtype=TORCH_DTYPE[wl.dtype], device=dw.device)
            self.bytes_written += self.bufs[n].numel() * self.bufs[n].element_size()

    def run(self, stream=None):
        wl = self.dw.wl
        tp = self.dw.table_ptrs()
        for n in self.order:
            op, ins, p = self.defs[n]
            vt.vt_copy_op(op, [(self.shapes[i], wl.dtype, self.bufs[i].data_ptr()) for i in ins], p, self.bufs[n],
                          stream=stream, tables=wl.index_tables, table_ptrs=tp)

    def identity_desc(self, name):
        return vt.build_chain([], {name: (self.shapes[name], self.dw.wl.dtype, self.bufs[name].data_ptr())}, name)


# ------------------------------------------------------------------------------------------
# C1: add + row-sum
# ------------------------------------------------------------------------------------------
class AddRowsum:
    def __init__(self, dw: DeviceWorkload, materialized=False):
        c = dw.wl.consumer
        self.dw = dw
        self.mat = Materialized(dw, [c["x"], c["y"]]) if materialized else None
        if materialized:
            self.x, self.y = self.mat.identity_desc(c["x"]), self.mat.identity_desc(c["y"])
        else:
            self.x, self.y = dw.build(c["x"]), dw.build(c["y"])
        self.out = torch.empty(self.x.shape[0], dtype=torch.float32, device=dw.device)

    def run(self, stream=None):
        if self.mat:
            self.mat.run(stream)
        vt.vt_elementwise(vt.EW_ADD_ROWSUM, self.x, self.y, 0.0, self.out, stream=stream)
        return self.out


# ------------------------------------------------------------------------------------------
# C2: decode attention
# ------------------------------------------------------------------------------------------
class DecodeAttention:
    def __init__(self, dw: DeviceWorkload, materialized=False, n_splits=0, want_lse=True):
        c = dw.wl.consumer
        self.dw = dw
        self.scale = float(c["scale"])
        self.n_splits = n_splits
        self.mat = Materialized(dw, [c["q"], c["k"], c["v"]]) if materialized else None
        if materialized:
            self.q, self.k, self.v = (self.mat.identity_desc(c[n]) for n in ("q", "k", "v"))
        else:
            self.q, self.k, self.v = (dw.build(c[n]) for n in ("q", "k", "v"))
        B, Hq, S, D = self.k.shape
        self.ws_bytes = vt.vt_decode_attn_workspace(B, Hq, D, S, n_splits)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dw.device)
        vt.vt_decode_attn_workspace_init(self.ws, self.ws_bytes)
        self.out = torch.empty((B, Hq, D), dtype=TORCH_DTYPE[dw.wl.dtype], device=dw.device)
        self.lse = torch.empty((B, Hq), dtype=torch.float32, device=dw.device) if want_lse else None

    def run(self, stream=None):
        if self.mat:
            self.mat.run(stream)
        vt.vt_decode_attn(self.q, self.k, self.v, self.scale, self.out, self.ws, self.ws_bytes, self.n_splits,
                          lse=self.lse, stream=stream)
        return self.out


def run_decode_attention(dw: DeviceWorkload, materialized=False, n_splits=0):
    p = DecodeAttention(dw, materialized, n_splits)
    p.run()
    torch.cuda.synchronize()
    return {"out": p.out, "lse": p.lse, "pipeline": p}


# ------------------------------------------------------------------------------------------
# C3 / C5: (grouped) GEMM;  C4: LayerNorm + linear
# ------------------------------------------------------------------------------------------
class Gemm:
    """consumer kinds "gemm" (one group), "grouped_gemm" (one group per expert, outputs stacked
    row-wise in one buffer) and "ln_linear" (LayerNorm prologue fused into the GEMM, or, with
    fused=False, the LayerNorm kernel followed by the GEMM on its dense result)."""

    def __init__(self, dw: DeviceWorkload, materialized=False, fused=True):
        c = dw.wl.consumer
        wl = dw.wl
        self.dw = dw
        kind = c["kind"]
        if kind == "gemm":
            a_names, b_names = [c["a"]], [c["b"]]
        elif kind == "grouped_gemm":
            a_names, b_names = list(c["a"]), list(c["b"])
        elif kind == "ln_linear":
            a_names, b_names = [c["x"]], [c["w"]]
        else:
            raise ValueError(kind)
        self.kind = kind
        self.eps = float(c.get("eps", 0.0))
        self.fused = fused
        self.mat = Materialized(dw, a_names + b_names) if materialized else None
        get = self.mat.identity_desc if materialized else dw.build
        self.A = [get(n) for n in a_names]
        self.B = [get(n) for n in b_names]
        rows = []
        for a in self.A:
            shp = a.shape
            r = 1
            for s in shp[:-1]:
                r *= s
            rows.append(r)
        self.N = self.B[0].shape[-1]
        self.rows = rows
        self.out = torch.empty((sum(rows), self.N), dtype=TORCH_DTYPE[wl.dtype], device=dw.device)
        self.C = []
        off = 0
        for r in rows:
            self.C.append(self.out.data_ptr() + off * self.N * self.out.element_size())
            off += r
        self.ln_buf = None
        if kind == "ln_linear" and not fused:
            shp = self.A[0].shape
            self.ln_buf = torch.empty(shp, dtype=TORCH_DTYPE[wl.dtype], device=dw.device)
            self.ln_desc = vt.build_chain([], {"ln": (shp, wl.dtype, self.ln_buf.data_ptr())}, "ln")

    def run(self, stream=None):
        if self.mat:
            self.mat.run(stream)
        dt = self.dw.wl.dtype
        if self.kind == "ln_linear":
            if self.fused:
                vt.vt_gemm(self.A, self.B, self.C, dt, vt.GEMM_LAYERNORM, self.eps, stream=stream)
            else:
                vt.vt_elementwise(vt.EW_LAYERNORM, self.A[0], None, self.eps, self.ln_buf, stream=stream)
                vt.vt_gemm([self.ln_desc], self.B, self.C, dt, vt.GEMM_PLAIN, 0.0, stream=stream)
        else:
            vt.vt_gemm(self.A, self.B, self.C, dt, vt.GEMM_PLAIN, 0.0, stream=stream)
        return self.out


# ------------------------------------------------------------------------------------------
# QKV projection with a producer-side store
# ------------------------------------------------------------------------------------------
class GemmStore:
    """consumer kind "gemm_store": the chain describes the OUTPUT.  virtual: one launch of
    vt_gemm_store writes the product through the output descriptor.  materialized: the same
    kernel writes the product to a dense buffer and a copy kernel scatters it to the physical
    targets (the Split / Reshape / ScatterND that the virtual store removes)."""

    def __init__(self, dw: DeviceWorkload, materialized=False):
        c = dw.wl.consumer
        wl = dw.wl
        self.dw = dw
        self.materialized = materialized
        self.A, self.B = dw.build(c["a"]), dw.build(c["b"])
        self.Cout = dw.build(c["out"])
        M, K = self.A.shape
        N = self.B.shape[1]
        self.shape = (M, N, K)
        self.ws_bytes = vt.vt_gemm_store_workspace(M, N, K)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dw.device)
        vt.vt_gemm_store_workspace_init(self.ws, self.ws_bytes)
        if materialized:
            self.dense = torch.empty((M, N), dtype=TORCH_DTYPE[wl.dtype], device=dw.device)
            self.dense_desc = vt.build_chain([], {"dense": ((M, N), wl.dtype, self.dense.data_ptr())}, "dense")

    def run(self, stream=None):
        if not self.materialized:
            vt.vt_gemm_store(self.A, self.B, self.Cout, self.ws, self.ws_bytes, stream=stream)
        else:
            # the same GEMM kernel into a dense buffer (identity descriptor), then the scatter
            vt.vt_gemm_store(self.A, self.B, self.dense_desc, self.ws, self.ws_bytes, stream=stream)
            vt.vt_scatter(self.dense_desc, self.Cout, stream=stream)
        return None


class WeightedSum:
    """consumer kind "weighted_sum" (mixture-of-experts combine): x and y are gathered through row
    tables; virtual: one launch reads the expert-major buffer in place; materialized: two gather
    copies, then the same consumer on the dense copies."""

    def __init__(self, dw: DeviceWorkload, materialized=False):
        c = dw.wl.consumer
        self.dw = dw
        self.mat = Materialized(dw, [c["x"], c["y"]]) if materialized else None
        get = self.mat.identity_desc if materialized else dw.build
        self.x, self.y = get(c["x"]), get(c["y"])
        self.w = torch.from_numpy(c["weights"]).to(dw.device)
        self.out = torch.empty(self.x.shape, dtype=TORCH_DTYPE[dw.wl.dtype], device=dw.device)

    def run(self, stream=None):
        if self.mat:
            self.mat.run(stream)
        vt.vt_weighted_sum(self.x, self.y, self.w, self.out, stream=stream)
        return self.out


class DecodeSegment:
    """Projection with a producer-side store followed by decode attention on the same buffers
    (Sec. 3.1 end to end).  virtual: two launches (vt_gemm_store, vt_decode_attn), no data
    movement operator is executed.  materialized: dense product + scatter, then every operator
    between the caches and the attention kernel as a copy."""

    def __init__(self, wl_store, wl_attn, materialized=False, device="cuda:0"):
        self.dw1 = DeviceWorkload(wl_store, device)
        self.dw2 = DeviceWorkload(wl_attn, device, share=self.dw1)
        self.store = GemmStore(self.dw1, materialized)
        self.attn = DecodeAttention(self.dw2, materialized)
        self.out, self.lse = self.attn.out, self.attn.lse

    def run(self, stream=None):
        self.store.run(stream)
        return self.attn.run(stream)


def make_pipeline(dw: DeviceWorkload, materialized=False, **kw):
    if dw.wl.consumer["kind"] == "gemm_store":
        return GemmStore(dw, materialized)
    if dw.wl.consumer["kind"] == "weighted_sum":
        return WeightedSum(dw, materialized)
    kind = dw.wl.consumer["kind"]
    if kind == "add_rowsum":
        return AddRowsum(dw, materialized)
    if kind == "decode_attn":
        return DecodeAttention(dw, materialized, **kw)
    return Gemm(dw, materialized, **kw)


# ------------------------------------------------------------------------------------------
# Profitability (Sec. 4.3) and the measured latency saving w(e) (Sec. 5.2) of one chain
# ------------------------------------------------------------------------------------------
def consumer_operands(p):
    """Descriptors the consumer of pipeline `p` reads."""
    if isinstance(p, (AddRowsum, WeightedSum)):
        return [p.x, p.y]
    if isinstance(p, DecodeAttention):
        return [p.q, p.k, p.v]
    return list(p.A) + list(p.B)


def time_pipeline(p, iters=20, warmup=3):
    """Mean microseconds per run of the launches `p.run()` makes, by HIP events on the current stream."""
    for _ in range(warmup):
        p.run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        p.run()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters


def choose_path(dw: DeviceWorkload, iters=20, warmup=3, unit_bytes=0, **kw):
    """Decide between reading the chain through descriptors and executing it as copies.

    The class of the chain is the worst class among the consumer's operands.  A fully contiguous
    chain is always profitable (Theorem 1) and is taken without measuring.  Any other chain is
    measured both ways, as the greedy search does for every candidate edge: the saving
    w = t(materialized) - t(virtual) decides, and a non-positive saving keeps the copies.
    Returns the chosen pipeline (ready to run) and a report."""
    virt = make_pipeline(dw, materialized=False, **kw)
    classes = [d.classify(unit_bytes) for d in consumer_operands(virt)]
    cls = max(c for c, _ in classes)
    report = {"class": ("full", "partial", "scattered")[cls], "min_run_bytes": min(r for _, r in classes)}
    if cls == vt.ACCESS_FULL:
        report.update(choice="virtual", measured=False)
        return virt, report
    mat = make_pipeline(dw, materialized=True, **kw)
    tv, tm = time_pipeline(virt, iters, warmup), time_pipeline(mat, iters, warmup)
    report.update(virtual_us=tv, materialized_us=tm, saving_us=tm - tv, measured=True,
                  choice="virtual" if tm - tv > 0 else "materialized")
    return (virt if tm - tv > 0 else mat), report


# ------------------------------------------------------------------------------------------
# A workload run under an arbitrary strategy of virtual tensors (Sec. 5): what the greedy search
# of vtog.py measures, and what it finally keeps
# ------------------------------------------------------------------------------------------
class StrategyPipeline:
    """`chosen` maps tensor names to opportunities (vtog.Opportunity): those tensors are virtual,
    in the read direction (the consumer reads through the map) or in the store direction: an input
    of a Concat is written straight into its range of the Concat's output, the input of a Reshape,
    Permute or Unsqueeze straight into that operator's output (through the inverse view).  Every
    other intermediate the consumer depends on is physical and is
    produced by one copy kernel that reads through the descriptor of the eliminated operators
    above it; the consumer reads its operands through descriptors over the nearest physical
    tensors.  With `chosen` empty this is the fully materialized path, with every tensor chosen
    the fully virtual one."""

    def __init__(self, dw: DeviceWorkload, chosen, statements=None, scatters=(), **kw):
        """`statements` replaces the workload's chain (same tensor names; used by lean_plan, which
        rewrites an append as a store).  `scatters`: (statement index, source tensor, statements
        that define the destination view over physical tensors, its name): executed with
        vt_scatter at that position, before the copies of later statements."""
        from . import vtog
        wl = dw.wl
        self.dw = dw
        stmts = list(statements if statements is not None else wl.chain)
        produced = {}
        for k, st in enumerate(stmts):
            for o in vtog.outputs_of(st):
                produced[o] = k
        self.consumer = make_pipeline(dw, materialized=False, **kw)
        operands = self._operand_names()
        self.bufs = {n: t for n, t in dw.tensors.items()}
        self.shapes = {n: tuple(t.shape) for n, t in dw.tensors.items()}
        self.copies = []           # (descriptor, destination buffer) in statement order
        self.bytes_written = 0
        read_opp = {}
        for st_i, st in enumerate(stmts):
            for o in vtog.outputs_of(st):
                read_opp[o] = vtog.Opportunity(o, tuple(i for i in st[2] if isinstance(i, str)), st_i, "read")
        done = set()
        # store direction (Sec. 4.2, Sec. 4.4): an input of a Concat that was made a virtual tensor
        # of the Concat's output is never stored on its own; it is written where it lives inside
        # the output.  Such a Concat is executed input by input: each one goes through its own map
        # (over whatever physical tensors it is made of) straight into its range of the output.
        stored = {t: o for t, o in chosen.items() if o.direction == "store"}
        bijective = ("reshape", "permute", "unsqueeze")
        for t, o in stored.items():
            if stmts[o.op_index][1] != "concat" and stmts[o.op_index][1] not in bijective:
                raise vt.VtError(vt.ERR_UNSUPPORTED, "store-direction choices are lowered for inputs of Concat, Reshape, Permute "
                                                     "and Unsqueeze (tensor %r is stored into a %s)" % (t, stmts[o.op_index][1]))
        chosen = {t: o for t, o in chosen.items() if o.direction == "read"}
        by_concat, by_bijective = {}, {}
        for t, o in stored.items():
            if stmts[o.op_index][1] == "concat":
                by_concat.setdefault(o.op_index, set()).add(t)
            else:
                by_bijective[o.op_index] = t

        # what a stored tensor holds is addressed through its producing operator (it has no buffer
        # of its own), also where one stored tensor is produced from another
        through_stored = dict(chosen)
        through_stored.update({t: read_opp[t] for t in stored if t in read_opp})

        def ensure(t):
            """make sure tensor t (a physical intermediate) has a buffer and a copy that fills it"""
            if t in done or t not in produced:
                return
            done.add(t)
            if produced[t] in by_concat:
                out, _, ins, p = stmts[produced[t]]
                dim = p["dim"]
                parts = []
                for i in ins:
                    via = through_stored if i in stored else dict(chosen)
                    chain, sources = vtog.read_chain(stmts, via, i)
                    for s in sources:
                        ensure(s)
                    parts.append(self._build(chain, sources, i))
                shape = list(parts[0].shape)
                shape[dim] = sum(d.shape[dim] for d in parts)
                self.shapes[t] = tuple(shape)
                self.bufs[t] = torch.empty(self.shapes[t], dtype=TORCH_DTYPE[wl.dtype], device=dw.device)
                self.bytes_written += self.bufs[t].numel() * self.bufs[t].element_size()
                at = 0
                for k, d in enumerate(parts):
                    slot = "%s__part%d" % (t, k)
                    dst = self._build([(slot, "slice", (t,), {"dim": dim, "start": at, "stop": at + d.shape[dim], "step": 1})], [t], slot)
                    self.copies.append((produced[t], d, dst))
                    at += d.shape[dim]
                return
            if produced[t] in by_bijective:
                # t = op(i) with i stored into t: what produces i is written through the inverse view
                # of t (i seen as a Reshape / Permute of t), so i never has a buffer of its own and
                # the operator between i and t is never executed
                _, kind, ins, p = stmts[produced[t]]
                i = ins[0]
                chain, sources = vtog.read_chain(stmts, through_stored, i)
                for s in sources:
                    ensure(s)
                src = self._build(chain, sources, i)
                ishape = tuple(src.shape)
                if kind == "permute":
                    perm = tuple(p["perm"])
                    tshape = tuple(ishape[j] for j in perm)
                    inverse = {"perm": tuple(sorted(range(len(perm)), key=lambda a: perm[a]))}
                    back = "permute"
                else:
                    n = 1
                    for e in ishape:
                        n *= e
                    tshape = tuple(p["shape"]) if kind == "reshape" else ishape[:p["dim"]] + (1,) + ishape[p["dim"]:]
                    if -1 in tshape:
                        known = 1
                        for e in tshape:
                            known *= e if e != -1 else 1
                        tshape = tuple(n // known if e == -1 else e for e in tshape)
                    inverse = {"shape": ishape}
                    back = "reshape"
                self.shapes[t] = tshape
                self.bufs[t] = torch.empty(tshape, dtype=TORCH_DTYPE[wl.dtype], device=dw.device)
                self.bytes_written += self.bufs[t].numel() * self.bufs[t].element_size()
                slot = "%s__as_%s" % (t, i)
                dst = self._build([(slot, back, (t,), inverse)], [t], slot)
                self.copies.append((produced[t], src, dst))
                return
            forced = dict(chosen)
            forced[t] = read_opp[t]
            chain, sources = vtog.read_chain(stmts, forced, t)
            for s in sources:
                ensure(s)
            d = self._build(chain, sources, t)
            self.shapes[t] = d.shape
            self.bufs[t] = torch.empty(d.shape, dtype=TORCH_DTYPE[wl.dtype], device=dw.device)
            self.bytes_written += self.bufs[t].numel() * self.bufs[t].element_size()
            self.copies.append((produced[t], d, self.bufs[t]))

        descs = []
        for name in operands:
            chain, sources = vtog.read_chain(stmts, chosen, name)
            for s in sources:
                ensure(s)
            descs.append(self._build(chain, sources, name))
        for index, src_name, dst_chain, dst_name in scatters:
            chain, sources = vtog.read_chain(stmts, chosen, src_name)
            for s in sources:
                ensure(s)
            src = self._build(chain, sources, src_name)
            dst_sources = sorted({i for st in dst_chain for i in st[2] if i in self.bufs})
            dst = self._build(list(dst_chain), dst_sources, dst_name)
            n = 1
            for e in src.shape:
                n *= e
            self.bytes_written += n * self.bufs[dst_sources[0]].element_size()
            self.copies.append((index, src, dst))
        self.copies.sort(key=lambda c: c[0])
        self._set_operands(descs)

    def _build(self, chain, sources, result):
        wl = self.dw.wl
        specs = {s: (self.shapes[s], wl.dtype, self.bufs[s].data_ptr()) for s in sources}
        return vt.build_chain(chain, specs, result, wl.index_tables, self.dw.table_ptrs())

    def _operand_names(self):
        c = self.dw.wl.consumer
        kind = c["kind"]
        if kind in ("add_rowsum", "weighted_sum"):
            return [c["x"], c["y"]]
        if kind == "decode_attn":
            return [c["q"], c["k"], c["v"]]
        if kind == "grouped_gemm":
            return list(c["a"]) + list(c["b"])
        if kind == "ln_linear":
            return [c["x"], c["w"]]
        return [c["a"], c["b"]]

    def _set_operands(self, descs):
        p = self.consumer
        if isinstance(p, (AddRowsum, WeightedSum)):
            p.x, p.y = descs
        elif isinstance(p, DecodeAttention):
            p.q, p.k, p.v = descs
        else:
            n = len(p.A)
            p.A, p.B = descs[:n], descs[n:]
        self.out = getattr(p, "out", None)

    def run(self, stream=None):
        for _, d, target in self.copies:
            if isinstance(target, vt.Desc):
                vt.vt_scatter(d, target, stream=stream)
            else:
                vt.vt_materialize(d, target, stream=stream)
        return self.consumer.run(stream)


VIEW_OPS = ("permute", "slice", "split", "unsqueeze", "expand")


def lean_plan(wl):
    """The chain as a stride-aware tensor framework executes it (the lean materialized comparison
    path): permute, slice, split, unsqueeze and expand return views; a reshape returns a view when
    the result is still one strided tensor and copies otherwise (after a permute or an expand);
    concat and index_select copy; a concat that puts new rows behind a leading slice of a graph
    input with room for them (a cache append) is executed in place: the new rows are stored into
    the input and the result is a view of it.
    Returns (statements, chosen, scatters) for StrategyPipeline: the tensors in `chosen` are views."""
    from . import vtog
    shapes = {k: tuple(v.shape) for k, v in wl.sources.items()}
    stmts, chosen, scatters = [], {}, []
    by_out = {}

    def desc_of(name):
        chain, sources = vtog.read_chain(stmts, chosen, name)
        return vt.build_chain(chain, {s_: (shapes[s_], wl.dtype) for s_ in sources}, name, wl.index_tables)

    for k, st in enumerate(wl.chain):
        out, op, ins, p = st
        if op == "concat" and len(ins) == 2 and ins[0] in by_out:
            head = stmts[by_out[ins[0]]]
            dim = p["dim"]
            if (head[1] == "slice" and head[2][0] in wl.sources and head[3]["dim"] == dim and head[3]["start"] == 0
                    and head[3].get("step", 1) == 1):
                base, pos = head[2][0], head[3]["stop"]
                ext = shapes[ins[1]][dim]
                if pos + ext <= shapes[base][dim]:
                    st = (out, "slice", (base,), {"dim": dim, "start": 0, "stop": pos + ext, "step": 1})
                    slot = out + "__slot"
                    scatters.append((k, ins[1], [(slot, "slice", (base,), {"dim": dim, "start": pos, "stop": pos + ext, "step": 1})], slot))
                    op = "slice"
        stmts.append(st)
        by_out[out] = len(stmts) - 1
        opp = vtog.Opportunity(out, tuple(i for i in st[2] if isinstance(i, str)), len(stmts) - 1, "read")
        if op in VIEW_OPS:
            chosen[out] = opp
        elif op == "reshape":
            chosen[out] = opp
            if desc_of(out).as_strided() is None:
                del chosen[out]
        shapes[out] = desc_of(out).shape if out in chosen else vt.build_chain(
            [st], {i: (shapes[i], wl.dtype) for i in st[2]}, out, wl.index_tables).shape
    return stmts, chosen, scatters


def make_lean_pipeline(dw: DeviceWorkload, **kw):
    """The lean materialized path of a workload: views stay views, the rest is copied (lean_plan)."""
    stmts, chosen, scatters = lean_plan(dw.wl)
    return StrategyPipeline(dw, chosen, statements=stmts, scatters=scatters, **kw)


def greedy_strategy(dw: DeviceWorkload, iters=10, warmup=2, **kw):
    """Alg. 2 with w(e) measured on the GPU: builds the opportunity graph of the workload's chain
    (read direction: the consumer-side opportunities this library can lower), times the workload
    under each candidate strategy, and returns (chosen, report)."""
    from . import vtog
    wl = dw.wl
    c = wl.consumer
    g = vtog.build_vtog(list(wl.chain), tuple(wl.sources), (), directions=("read",))
    times = {}

    def latency(chosen):
        key = frozenset((t, o.op_index) for t, o in chosen.items())
        if key not in times:
            try:
                p = StrategyPipeline(dw, chosen, **kw)
                times[key] = time_pipeline(p, iters, warmup)
                del p
            except vt.VtError as e:
                # a layout the consumer kernel does not take is not an opportunity on this machine
                if e.code != vt.ERR_UNSUPPORTED:
                    raise
                times[key] = float("inf")
            torch.cuda.empty_cache()
        return times[key]

    def profile(o, chosen):
        grown = dict(chosen)
        grown[o.tensor] = o
        t0, t1 = latency(chosen), latency(grown)
        return float("-inf") if t1 == float("inf") else t0 - t1

    chosen, total, trace = vtog.greedy(g, profile)
    report = {"all_physical_us": latency({}), "chosen_us": latency(chosen), "saving_us": total,
              "virtual_tensors": [o.tensor for o, _ in trace], "strategies_timed": len(times),
              "opportunities": len(g.opportunities)}
    return chosen, report
