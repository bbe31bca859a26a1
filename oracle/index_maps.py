"""Per-operator mapping functions F(i, x) = (j, y) (Def. 2) in pure Python, and a
brute-force materializer that enumerates every output index.

These are the operator definitions written out one index at a time; they are used on
tiny tensors to pin the dense numpy routines in ``dm_ops`` and, composed backwards along
a chain (``pull_back``), to give for any virtual index the source tensor and the source
index it comes from (Def. 3: V = (F, {P_1..P_n}); composition F_new = F_outer ∘ F_base).

Operator semantics follow ONNX (the paper's stated authority for operator definitions);
for Transpose the ONNX convention out.shape[i] = in.shape[perm[i]] is used (the paper's
Def. 1 prints the inverse convention; the benchmark's chains are written for ONNX's).
"""
from __future__ import annotations

import itertools

import numpy as np


def out_shape(op, in_shapes, p, tables=None):
    """Shape of the output named by the statement (for split: output p['output'])."""
    s = tuple(in_shapes[0])
    if op == "permute":
        return tuple(s[a] for a in p["perm"])
    if op == "reshape":
        new = tuple(int(v) for v in p["shape"])
        assert int(np.prod(new, dtype=np.int64)) == int(np.prod(s, dtype=np.int64)), (s, new)
        return new
    if op == "slice":
        d, st, sp, step = p["dim"], p["start"], p["stop"], p.get("step", 1)
        assert 0 <= st < sp <= s[d] and step >= 1
        return s[:d] + ((sp - st + step - 1) // step,) + s[d + 1:]
    if op == "split":
        d = p["dim"]
        assert sum(p["sizes"]) == s[d]
        return s[:d] + (p["sizes"][p["output"]],) + s[d + 1:]
    if op == "concat":
        d = p["dim"]
        for t in in_shapes:
            assert tuple(t[:d]) == s[:d] and tuple(t[d + 1:]) == s[d + 1:]
        return s[:d] + (sum(t[d] for t in in_shapes),) + s[d + 1:]
    if op == "unsqueeze":
        d = p["dim"]
        return s[:d] + (1,) + s[d:]
    if op == "expand":
        new = tuple(int(v) for v in p["shape"])
        assert len(new) == len(s)
        for a, b in zip(s, new):
            assert a == b or a == 1
        return new
    if op == "index_select":
        d = p["dim"]
        return s[:d] + (len(tables[p["index"]]),) + s[d + 1:]
    raise ValueError(op)


def F(op, in_shapes, p, x, tables=None):
    """Output index x -> (input number j, input index y)."""
    x = tuple(int(v) for v in x)
    s = tuple(in_shapes[0])
    if op == "permute":
        y = [0] * len(x)
        for i, a in enumerate(p["perm"]):
            y[a] = x[i]                      # output dim i is input dim perm[i]
        return 0, tuple(y)
    if op == "reshape":
        new = out_shape(op, in_shapes, p)
        lin = 0
        for xi, di in zip(x, new):           # row-major linear index is preserved
            lin = lin * di + xi
        y = []
        for di in reversed(s):
            y.append(lin % di)
            lin //= di
        return 0, tuple(reversed(y))
    if op == "slice":
        d = p["dim"]
        return 0, x[:d] + (p["start"] + p.get("step", 1) * x[d],) + x[d + 1:]
    if op == "split":
        d = p["dim"]
        off = sum(p["sizes"][:p["output"]])
        return 0, x[:d] + (x[d] + off,) + x[d + 1:]
    if op == "concat":
        d = p["dim"]
        pos = x[d]
        for j, t in enumerate(in_shapes):
            if pos < t[d]:
                return j, x[:d] + (pos,) + x[d + 1:]
            pos -= t[d]
        raise IndexError(x)
    if op == "unsqueeze":
        d = p["dim"]
        return 0, x[:d] + x[d + 1:]
    if op == "expand":
        return 0, tuple(0 if a == 1 else xi for xi, a in zip(x, s))
    if op == "index_select":
        d = p["dim"]
        return 0, x[:d] + (int(tables[p["index"]][x[d]]),) + x[d + 1:]
    raise ValueError(op)


def materialize_bruteforce(op, inputs, p, tables=None):
    """O[x] = I_j[F(x)] for every x, one element at a time."""
    in_shapes = [a.shape for a in inputs]
    shp = out_shape(op, in_shapes, p, tables)
    out = np.empty(shp, dtype=inputs[0].dtype)
    for x in itertools.product(*[range(n) for n in shp]):
        j, y = F(op, in_shapes, p, x, tables)
        out[x] = inputs[j][y]
    return out


class Chain:
    """Shape inference over a chain and backwards evaluation of the composed map."""

    def __init__(self, chain, source_shapes, tables=None):
        self.tables = tables or {}
        self.shapes = {k: tuple(v) for k, v in source_shapes.items()}
        self.defs = {}
        for out, op, ins, p in chain:
            self.shapes[out] = out_shape(op, [self.shapes[i] for i in ins], p, self.tables)
            self.defs[out] = (op, ins, p)

    def pull_back(self, name, x):
        """Virtual index x of value `name` -> (source name, source index)."""
        x = tuple(int(v) for v in x)
        while name in self.defs:
            op, ins, p = self.defs[name]
            j, x = F(op, [self.shapes[i] for i in ins], p, x, self.tables)
            name = ins[j]
        return name, x

    def materialize_by_pull_back(self, name, sources):
        shp = self.shapes[name]
        first = next(iter(sources.values()))
        out = np.empty(shp, dtype=first.dtype)
        for x in itertools.product(*[range(n) for n in shp]):
            s, y = self.pull_back(name, x)
            out[x] = sources[s][y]
        return out
