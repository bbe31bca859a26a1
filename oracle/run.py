"""Run a whole workload on the CPU: every data-movement statement into a dense array, then
the consumer.  The workload object carries only shapes, stored bits and statements."""
from __future__ import annotations

import numpy as np

from . import consumers, dm_ops


def run_workload(wl, keep_intermediates: bool = False):
    """Returns a dict: 'out' (float64 or, for add_rowsum, float32), extra keys per consumer."""
    c = wl.consumer
    kind = c["kind"]
    if kind == "gemm_store":
        # the chain describes the OUTPUT here: the product of two physical operands, rounded to
        # the storage type, is assigned to the virtual tensor the chain defines
        a = consumers.decode(wl.sources[c["a"]], wl.dtype)
        b = consumers.decode(wl.sources[c["b"]], wl.dtype)
        out = consumers.gemm(a, b)
        return {"out": out, "stored": dm_ops.store_through(wl.chain, wl.sources, c["out"],
                                                           consumers.round_to(out, wl.dtype), wl.index_tables)}
    if kind == "grouped_gemm":
        wanted = set(c["a"]) | set(c["b"])
    else:
        wanted = {c[k] for k in ("x", "y", "q", "k", "v", "a", "b", "w") if k in c and isinstance(c[k], str)}
    env = dm_ops.run_chain(wl.chain, wl.sources, wl.index_tables,
                           keep=None if keep_intermediates else wanted)
    dec = lambda name: consumers.decode(env[name], wl.dtype)   # noqa: E731
    res = {}
    if kind == "materialize":
        res["out"] = env[c["x"]]
    elif kind == "add_rowsum":
        res["out"] = consumers.add_rowsum_f32(env[c["x"]], env[c["y"]])
        res["out_f64"] = (dec(c["x"]) + dec(c["y"])).sum(axis=1)
    elif kind == "gemm":
        res["out"] = consumers.gemm(dec(c["a"]), dec(c["b"]))
    elif kind == "grouped_gemm":
        res["out"] = np.concatenate(
            [consumers.gemm(dec(a), dec(b)) for a, b in zip(c["a"], c["b"])], axis=0)
    elif kind == "ln_linear":
        res["out"] = consumers.ln_linear(dec(c["x"]), dec(c["w"]), c["eps"], wl.dtype)
        res["ln"] = consumers.layernorm(dec(c["x"]), c["eps"])
    elif kind == "weighted_sum":
        res["out"] = consumers.weighted_sum(dec(c["x"]), dec(c["y"]), c["weights"])
    elif kind == "decode_attn":
        out, lse = consumers.decode_attention(dec(c["q"]), dec(c["k"]), dec(c["v"]), c["scale"])
        res["out"], res["lse"] = out, lse
    else:
        raise ValueError(kind)
    if keep_intermediates:
        res["env"] = env
    return res
