"""ctypes binding over libvt.so: argument marshalling only.

Every step of the hot path runs inside the library's kernels; this module turns Python
objects (shapes, statement tuples, torch tensors used as device memory) into the C structs
of include/vt.h.  If the library has not been built it raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("VT_LIB_PATH", os.path.join(HERE, "libvt.so"))   # override: kernel experiments

VT_MAX_DIMS = 8
VT_MAX_OP_INPUTS = 8

OK, ERR_INVALID_ARG, ERR_SHAPE, ERR_RANGE, ERR_NOT_ONE_TO_ONE, ERR_UNSUPPORTED, ERR_DEVICE = range(7)
F32, F16, BF16 = 0, 1, 2
DTYPES = {"f32": F32, "f16": F16, "bf16": BF16}
OP_KINDS = {"reshape": 0, "permute": 1, "slice": 2, "split": 3, "concat": 4, "expand": 5,
            "unsqueeze": 6, "index_select": 7}
EW_ADD_ROWSUM, EW_LAYERNORM = 0, 1
GEMM_PLAIN, GEMM_LAYERNORM = 0, 1
ACCESS_FULL, ACCESS_PARTIAL, ACCESS_SCATTERED = 0, 1, 2


class VtSource(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32), ("ndim", C.c_int32),
                ("shape", C.c_int64 * VT_MAX_DIMS), ("stride", C.c_int64 * VT_MAX_DIMS)]


class VtOp(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_in", C.c_int32), ("in_", C.c_int32 * VT_MAX_OP_INPUTS),
                ("out_index", C.c_int32), ("ndim", C.c_int32),
                ("a", C.c_int64 * VT_MAX_DIMS), ("b", C.c_int64 * VT_MAX_DIMS),
                ("index", C.c_void_p), ("index_host", C.c_void_p), ("n_index", C.c_int64)]


class VtGraphStmt(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_in", C.c_int32), ("in_", C.c_int32 * VT_MAX_OP_INPUTS),
                ("n_out", C.c_int32), ("out", C.c_int32 * VT_MAX_OP_INPUTS)]


SAVING_FN = C.CFUNCTYPE(C.c_double, C.c_void_p, C.c_int, C.POINTER(C.c_int))
OP_SCATTER_ND, OP_COMPUTE, DIR_READ, DIR_STORE = 8, -1, 1, 2


class VtError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("vt error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libvt.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback for the hot path)")
        L = C.CDLL(LIB_PATH)
        P = C.c_void_p
        L.vt_build.argtypes = [C.POINTER(VtSource), C.c_int, C.POINTER(VtOp), C.c_int, C.c_int, C.POINTER(P)]
        L.vt_free.argtypes = [P]
        L.vt_desc_info.argtypes = [P, C.POINTER(C.c_int), C.POINTER(C.c_int64), C.POINTER(C.c_int),
                                   C.POINTER(C.c_int64), C.POINTER(C.c_int)]
        L.vt_desc_piece.argtypes = [P, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int),
                                    C.POINTER(C.c_int64)]
        L.vt_classify.argtypes = [P, C.c_int64, C.POINTER(C.c_int), C.POINTER(C.c_int64)]
        L.vt_desc_block.argtypes = [P, C.c_int64, C.POINTER(C.c_int64)]
        L.vt_desc_as_strided.argtypes = [P, C.POINTER(C.c_int), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.vt_desc_row_walk.argtypes = [P, C.c_int64, C.POINTER(C.c_int), C.POINTER(C.c_int64)]
        L.vt_desc_walk_addresses.argtypes = [P, C.c_int64, C.c_int64, C.c_int64, C.POINTER(C.c_int), C.POINTER(C.c_uint64)]
        L.vt_eval_host.argtypes = [P, C.POINTER(C.c_int64), C.POINTER(C.c_int), C.POINTER(C.c_int64)]
        L.vt_eval_device_form.argtypes = [P, C.POINTER(C.c_int64), C.POINTER(C.c_int), C.POINTER(C.c_int64)]
        L.vt_desc_dump.argtypes = [P, C.c_char_p, C.c_size_t]
        L.vt_materialize.argtypes = [P, P, P]
        L.vt_copy_op.argtypes = [C.POINTER(VtSource), C.c_int, C.POINTER(VtOp), P, P]
        L.vt_elementwise.argtypes = [C.c_int, P, P, C.c_float, P, P]
        L.vt_gemm.argtypes = [C.POINTER(P), C.POINTER(P), C.POINTER(P), C.c_int, C.c_int, C.c_int, C.c_float, P]
        L.vt_scatter.argtypes = [P, P, P]
        L.vt_weighted_sum.argtypes = [P, P, P, P, P]
        L.vt_gemm_store_workspace.argtypes = [C.c_int64, C.c_int64, C.c_int64]
        L.vt_gemm_store_workspace.restype = C.c_size_t
        L.vt_gemm_store_workspace_init.argtypes = [P, C.c_size_t, P]
        L.vt_gemm_store.argtypes = [P, P, P, P, C.c_size_t, P]
        L.vt_decode_attn_plan.argtypes = [P, P, P, C.c_int] + [C.POINTER(C.c_int)] * 4
        L.vt_decode_attn_workspace.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
        L.vt_decode_attn_workspace.restype = C.c_size_t
        L.vt_decode_attn_workspace_init.argtypes = [P, C.c_size_t, P]
        L.vt_decode_attn.argtypes = [P, P, P, C.c_float, P, P, P, C.c_size_t, C.c_int, P]
        L.vt_decode_attn_static_capacity.argtypes = []
        L.vt_decode_attn_static_capacity.restype = C.c_size_t
        L.vt_decode_attn_static.argtypes = [P, P, P, C.c_float, P, P, C.c_int, P]
        L.vt_vtog_build.argtypes = [C.POINTER(VtGraphStmt), C.c_int, C.c_int, C.POINTER(C.c_uint8), C.c_int, C.POINTER(P)]
        L.vt_vtog_free.argtypes = [P]
        L.vt_vtog_size.argtypes = [P, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.vt_vtog_bundle.argtypes = [P, C.c_int] + [C.POINTER(C.c_int)] * 5
        L.vt_vtog_is_points_to_graph.argtypes = [P, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.vt_vtog_greedy.argtypes = [P, SAVING_FN, C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_double), C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.vt_last_error.restype = C.c_char_p
        L.vt_version.restype = C.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != OK:
        raise VtError(rc, lib().vt_last_error().decode())


def make_source(shape, dtype, ptr=0, stride=None) -> VtSource:
    s = VtSource()
    s.ptr = int(ptr) if ptr else None
    s.dtype = DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
    s.ndim = len(shape)
    for i, n in enumerate(shape):
        s.shape[i] = int(n)
        s.stride[i] = int(stride[i]) if stride is not None else 0
    return s


def make_op(op: str, in_ids, p: dict, tables=None, table_ptrs=None, keep=None) -> VtOp:
    """One statement.  in_ids are value ids (see vt.h).  For index_select, `tables[name]` is the
    host int32 array and `table_ptrs[name]` the device address (0 if the descriptor is only
    evaluated on the host).  `keep` collects objects that must outlive the call."""
    o = VtOp()
    o.kind = OP_KINDS[op]
    o.n_in = len(in_ids)
    for i, v in enumerate(in_ids):
        o.in_[i] = int(v)
    if op in ("reshape", "expand"):
        o.ndim = len(p["shape"])
        for i, n in enumerate(p["shape"]):
            o.a[i] = int(n)
    elif op == "permute":
        o.ndim = len(p["perm"])
        for i, n in enumerate(p["perm"]):
            o.a[i] = int(n)
    elif op == "slice":
        o.a[0], o.a[1], o.a[2], o.a[3] = int(p["dim"]), int(p["start"]), int(p["stop"]), int(p.get("step", 1))
    elif op == "split":
        o.a[0] = int(p["dim"])
        o.ndim = len(p["sizes"])
        for i, n in enumerate(p["sizes"]):
            o.b[i] = int(n)
        o.out_index = int(p["output"])
    elif op in ("concat", "unsqueeze"):
        o.a[0] = int(p["dim"])
    elif op == "index_select":
        o.a[0] = int(p["dim"])
        host = np.ascontiguousarray(tables[p["index"]], dtype=np.int32)
        if keep is not None:
            keep.append(host)
        o.index_host = host.ctypes.data
        o.n_index = host.size
        dev = (table_ptrs or {}).get(p["index"], 0)
        o.index = int(dev) if dev else None
    else:
        raise ValueError(op)
    return o


class Desc:
    """Owns a vt_desc*."""

    def __init__(self, handle, keep=None):
        self.handle = C.c_void_p(handle)
        self._keep = keep

    def __del__(self):
        try:
            if self.handle:
                lib().vt_free(self.handle)
                self.handle = None
        except Exception:
            pass

    def info(self):
        nd, dt, run, npc = C.c_int(), C.c_int(), C.c_int64(), C.c_int()
        shp = (C.c_int64 * VT_MAX_DIMS)()
        _check(lib().vt_desc_info(self.handle, C.byref(nd), shp, C.byref(dt), C.byref(run), C.byref(npc)))
        return {"shape": tuple(shp[i] for i in range(nd.value)), "dtype": dt.value, "run": run.value,
                "n_pieces": npc.value}

    @property
    def shape(self):
        return self.info()["shape"]

    def classify(self, unit_bytes=0):
        """(class, shortest run in bytes); class is ACCESS_FULL / ACCESS_PARTIAL / ACCESS_SCATTERED."""
        cls, run = C.c_int(), C.c_int64()
        _check(lib().vt_classify(self.handle, unit_bytes, C.byref(cls), C.byref(run)))
        return cls.value, run.value

    def block(self, cap_elems=1 << 20):
        """Largest power-of-two block (elements, <= cap) that is contiguous in one source wherever it is aligned."""
        out = C.c_int64()
        _check(lib().vt_desc_block(self.handle, cap_elems, C.byref(out)))
        return out.value

    def as_strided(self):
        """(strides, offset) in elements if the map is a plain strided view of one tensor, else None."""
        flag, off = C.c_int(), C.c_int64()
        st = (C.c_int64 * VT_MAX_DIMS)()
        _check(lib().vt_desc_as_strided(self.handle, C.byref(flag), st, C.byref(off)))
        if not flag.value:
            return None
        return tuple(st[i] for i in range(len(self.shape))), off.value

    def row_walk(self, block_elems):
        """Segments in which the block address of a [R, C] map is affine in the row and in at most two levels of
        the block index: a list of (row_lo, row_hi, blk_lo, blk_hi, address, row_stride_bytes, blk_stride_bytes,
        blk_group, group_stride_bytes); empty if the map has another form."""
        n = C.c_int()
        seg = (C.c_int64 * 36)()
        _check(lib().vt_desc_row_walk(self.handle, block_elems, C.byref(n), seg))
        return [tuple(seg[9 * k + i] for i in range(9)) for k in range(n.value)]

    def walk_addresses(self, unit_elems, first=0, count=None):
        """Addresses of the units [first, first + count) of unit_elems elements each, computed from the map's
        resolved term form (the kernels' own routine, run on the host); None if the map does not resolve."""
        n = 1
        for e in self.shape:
            n *= e
        if count is None:
            count = n // unit_elems - first if unit_elems > 0 else 0
        flag = C.c_int()
        buf = (C.c_uint64 * max(count, 1))()
        _check(lib().vt_desc_walk_addresses(self.handle, unit_elems, first, count, C.byref(flag), buf))
        if not flag.value:
            return None
        return [buf[i] for i in range(count)]

    def piece(self, p):
        lo, hi = (C.c_int64 * VT_MAX_DIMS)(), (C.c_int64 * VT_MAX_DIMS)()
        src, run = C.c_int(), C.c_int64()
        _check(lib().vt_desc_piece(self.handle, p, lo, hi, C.byref(src), C.byref(run)))
        n = len(self.shape)
        return {"lo": tuple(lo[i] for i in range(n)), "hi": tuple(hi[i] for i in range(n)), "src": src.value,
                "run": run.value}

    def eval_host(self, index):
        v = (C.c_int64 * VT_MAX_DIMS)(*[int(i) for i in index])
        src, off = C.c_int(), C.c_int64()
        _check(lib().vt_eval_host(self.handle, v, C.byref(src), C.byref(off)))
        return src.value, off.value

    def eval_device_form(self, index):
        v = (C.c_int64 * VT_MAX_DIMS)(*[int(i) for i in index])
        pc, off = C.c_int(), C.c_int64()
        _check(lib().vt_eval_device_form(self.handle, v, C.byref(pc), C.byref(off)))
        return pc.value, off.value

    def dump(self):
        buf = C.create_string_buffer(8192)
        _check(lib().vt_desc_dump(self.handle, buf, 8192))
        return buf.value.decode()


def build_raw(sources, ops, result_value, keep=None) -> Desc:
    sa = (VtSource * len(sources))(*sources)
    oa = (VtOp * max(1, len(ops)))(*ops) if ops else None
    out = C.c_void_p()
    _check(lib().vt_build(sa, len(sources), oa, len(ops), result_value, C.byref(out)))
    return Desc(out.value, keep)


def build_chain(chain, source_specs: dict, result: str, tables=None, table_ptrs=None) -> Desc:
    """Build the descriptor of value `result` of a chain written as statement tuples.
    source_specs: name -> (shape, dtype[, ptr[, stride]]).  Only the statements that `result`
    depends on are handed to the library; source numbers follow first use."""
    defs = {out: (op, ins, p) for out, op, ins, p in chain}
    order, seen = [], set()

    def visit(name):
        if name in seen or name not in defs:
            return
        seen.add(name)
        for i in defs[name][1]:
            visit(i)
        order.append(name)

    visit(result)
    src_ids, sources = {}, []

    def value_id(name):
        if name in defs:
            return order.index(name)
        if name not in src_ids:
            spec = source_specs[name]
            src_ids[name] = len(sources)
            sources.append(make_source(*spec))
        return -1 - src_ids[name]

    keep, ops = [], []
    for name in order:
        op, ins, p = defs[name]
        ops.append(make_op(op, [value_id(i) for i in ins], p, tables, table_ptrs, keep))
    rv = value_id(result)
    d = build_raw(sources, ops, rv, keep)
    d.source_names = [n for n, _ in sorted(src_ids.items(), key=lambda kv: kv[1])]
    return d


def _ptr(t):
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return C.c_void_p(t.data_ptr())
    return C.c_void_p(int(t))


def _stream(stream):
    if stream is None:
        try:
            import torch
            return C.c_void_p(torch.cuda.current_stream().cuda_stream)
        except Exception:
            return None
    if hasattr(stream, "cuda_stream"):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


def vt_materialize(desc: Desc, dst, stream=None):
    _check(lib().vt_materialize(desc.handle, _ptr(dst), _stream(stream)))


def vt_copy_op(op: str, inputs, p: dict, dst, stream=None, tables=None, table_ptrs=None):
    """inputs: list of (shape, dtype, ptr[, stride])."""
    keep = []
    srcs = (VtSource * len(inputs))(*[make_source(*spec) for spec in inputs])
    o = make_op(op, [-1 - i for i in range(len(inputs))], p, tables, table_ptrs, keep)
    _check(lib().vt_copy_op(srcs, len(inputs), C.byref(o), _ptr(dst), _stream(stream)))


def vt_elementwise(kind: int, x: Desc, y, eps: float, out, stream=None):
    _check(lib().vt_elementwise(kind, x.handle, y.handle if y is not None else None, C.c_float(eps), _ptr(out),
                                _stream(stream)))


def vt_gemm(A, B, Cs, c_dtype, prologue=GEMM_PLAIN, eps=0.0, stream=None):
    """A, B: lists of Desc (one per group); Cs: list of device tensors / addresses."""
    n = len(A)
    assert len(B) == n and len(Cs) == n
    P = C.c_void_p
    a = (P * n)(*[d.handle for d in A])
    b = (P * n)(*[d.handle for d in B])
    c = (P * n)(*[_ptr(t) for t in Cs])
    dt = DTYPES[c_dtype] if isinstance(c_dtype, str) else int(c_dtype)
    _check(lib().vt_gemm(a, b, c, n, dt, int(prologue), C.c_float(eps), _stream(stream)))


def vt_decode_attn_workspace(B, Hq, D, S, n_splits=0) -> int:
    return int(lib().vt_decode_attn_workspace(B, Hq, D, S, n_splits))


def vt_decode_attn_workspace_init(workspace, workspace_bytes: int, stream=None):
    _check(lib().vt_decode_attn_workspace_init(_ptr(workspace), workspace_bytes, _stream(stream)))


def vt_decode_attn(Q: Desc, K: Desc, V: Desc, scale: float, out, workspace, workspace_bytes: int, n_splits=0,
                   lse=None, stream=None):
    _check(lib().vt_decode_attn(Q.handle, K.handle, V.handle, C.c_float(scale), _ptr(out), _ptr(lse),
                                _ptr(workspace), workspace_bytes, n_splits, _stream(stream)))


def vt_decode_attn_static_capacity() -> int:
    return int(lib().vt_decode_attn_static_capacity())


def vt_decode_attn_static(Q: Desc, K: Desc, V: Desc, scale: float, out, n_splits=0, lse=None, stream=None):
    _check(lib().vt_decode_attn_static(Q.handle, K.handle, V.handle, C.c_float(scale), _ptr(out), _ptr(lse),
                                       n_splits, _stream(stream)))


def vt_gemm_store_workspace(M, N, K) -> int:
    return int(lib().vt_gemm_store_workspace(M, N, K))


def vt_gemm_store_workspace_init(workspace, workspace_bytes: int, stream=None):
    _check(lib().vt_gemm_store_workspace_init(_ptr(workspace), workspace_bytes, _stream(stream)))


def vt_gemm_store(A: Desc, B: Desc, Cout: Desc, workspace, workspace_bytes: int, stream=None):
    _check(lib().vt_gemm_store(A.handle, B.handle, Cout.handle, _ptr(workspace), workspace_bytes, _stream(stream)))


def vt_scatter(src: Desc, dst: Desc, stream=None):
    _check(lib().vt_scatter(src.handle, dst.handle, _stream(stream)))


def vt_decode_attn_plan(Q: Desc, K: Desc, V: Desc, n_splits=0):
    """Host-side plan of vt_decode_attn: dict with group_size, n_segments, splits, paged_segments."""
    g, ns, sp, pg = C.c_int(), C.c_int(), C.c_int(), C.c_int()
    _check(lib().vt_decode_attn_plan(Q.handle, K.handle, V.handle, n_splits, C.byref(g), C.byref(ns), C.byref(sp), C.byref(pg)))
    return {"group_size": g.value, "n_segments": ns.value, "splits": sp.value, "paged_segments": pg.value}


def vt_weighted_sum(x: Desc, y: Desc, weights, out, stream=None):
    _check(lib().vt_weighted_sum(x.handle, y.handle, _ptr(weights), _ptr(out), _stream(stream)))
