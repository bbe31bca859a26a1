"""Dense execution of data-movement operators: each call returns a fresh contiguous
row-major array (the "materialized" intermediate the paper's method avoids writing).

Each routine is the operator's definition (Def. 2; ONNX semantics) expressed with the
numpy primitive of the same meaning and then copied into new memory.  They operate on
the stored bits (float32 / float16 / uint16-for-bf16), so data movement is exact.  They
are pinned on tiny tensors against ``index_maps.materialize_bruteforce``.
"""
from __future__ import annotations

import numpy as np


def permute(x, perm):
    # ONNX Transpose: out.shape[i] = in.shape[perm[i]]
    return np.ascontiguousarray(np.transpose(x, perm))


def reshape(x, shape):
    # row-major linear order is preserved (Sec. 2.1 stride vector of a dense tensor)
    return np.array(np.reshape(np.ascontiguousarray(x), shape, order="C"), copy=True)


def slice_(x, dim, start, stop, step=1):
    idx = [slice(None)] * x.ndim
    idx[dim] = slice(start, stop, step)
    return np.ascontiguousarray(x[tuple(idx)])


def split(x, dim, sizes):
    assert sum(sizes) == x.shape[dim]
    outs, off = [], 0
    for n in sizes:
        outs.append(slice_(x, dim, off, off + n, 1))
        off += n
    return outs


def concat(xs, dim):
    return np.ascontiguousarray(np.concatenate(xs, axis=dim))


def unsqueeze(x, dim):
    return np.array(np.expand_dims(x, dim), copy=True)


def expand(x, shape):
    # ONNX Expand restricted to same rank: size-1 dims broadcast
    return np.ascontiguousarray(np.broadcast_to(x, shape))


def index_select(x, dim, index):
    return np.ascontiguousarray(np.take(x, np.asarray(index, dtype=np.int64), axis=dim))


def run_statement(op, inputs, p, tables=None):
    if op == "permute":
        return permute(inputs[0], p["perm"])
    if op == "reshape":
        return reshape(inputs[0], p["shape"])
    if op == "slice":
        return slice_(inputs[0], p["dim"], p["start"], p["stop"], p.get("step", 1))
    if op == "split":
        return split(inputs[0], p["dim"], p["sizes"])[p["output"]]
    if op == "concat":
        return concat(list(inputs), p["dim"])
    if op == "unsqueeze":
        return unsqueeze(inputs[0], p["dim"])
    if op == "expand":
        return expand(inputs[0], p["shape"])
    if op == "index_select":
        return index_select(inputs[0], p["dim"], tables[p["index"]])
    raise ValueError(op)


def run_chain(chain, sources, tables=None, keep=None):
    """Execute every statement in order; returns {name: dense array}.  ``keep`` limits which
    intermediates are retained (names), to bound memory on the large configurations."""
    env = dict(sources)
    last_use = {}
    for k, (_, _, ins, _) in enumerate(chain):
        for i in ins:
            last_use[i] = k
    for k, (out, op, ins, p) in enumerate(chain):
        env[out] = run_statement(op, [env[i] for i in ins], p, tables)
        if keep is not None:
            for i in ins:
                if last_use[i] == k and i not in keep and i not in sources:
                    env.pop(i, None)
    return env


def store_through(chain, sources, name, values, tables=None):
    """Producer-side store (Sec. 4.2, the write direction of Def. 2): the virtual tensor `name`
    is assigned `values`; every element lands in the physical tensor and at the index that the
    chain's map names, and everything else keeps what it held (the result of a ScatterND is a
    clone of its data input with the updates written in, Sec. 4.4).  The map must be one to one
    on the elements it reaches: two virtual elements on one physical element is an error.

    Returns updated copies of the sources that were written (others are not returned)."""
    from .index_maps import Chain
    import itertools
    ch = Chain(chain, {k: v.shape for k, v in sources.items()}, tables)
    shp = ch.shapes[name]
    values = np.asarray(values)
    assert values.shape == shp, (values.shape, shp)
    out, seen = {}, set()
    for x in itertools.product(*[range(n) for n in shp]):
        s, y = ch.pull_back(name, x)
        if (s, y) in seen:
            raise ValueError("store through a map that is not one to one: %s%s written twice" % (s, y))
        seen.add((s, y))
        if s not in out:
            out[s] = sources[s].copy()
        out[s][y] = values[x]
    return out
