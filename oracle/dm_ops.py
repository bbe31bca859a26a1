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
