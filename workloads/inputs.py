"""Seeded input generators and chain descriptions for the benchmark configurations.

A chain is a list of statements ``(out, op, inputs, params)``:

    ("t1", "permute",      ("X",),      {"perm": (2, 0, 1)})
    ("t2", "reshape",      ("t1",),     {"shape": (8, 24)})
    ("t3", "slice",        ("t2",),     {"dim": 1, "start": 4, "stop": 20, "step": 1})
    ("q",  "split",        ("x",),      {"dim": 2, "sizes": (4096, 1024, 1024), "output": 0})
    ("V",  "concat",       ("t3", "Y"), {"dim": 1})
    ("u",  "unsqueeze",    ("k",),      {"dim": 2})
    ("e",  "expand",       ("u",),      {"shape": (8, 8, 4, 4096, 128)})
    ("a",  "index_select", ("tok",),    {"dim": 0, "index": "idx0"})

Names that are not produced by an earlier statement refer to ``sources`` (or, for
``index``, to ``index_tables``).  Every value is generated on the host from
``numpy.random.Generator(PCG64)`` streams keyed by ``(seed, tensor number)``, in
float32, and then rounded once (round-to-nearest-even) to the storage type; the
stored bits are what both the oracle and the GPU path consume.

Storage: "f32" -> float32 arrays, "f16" -> float16 arrays, "bf16" -> uint16 arrays
holding the upper half of the float32 bit pattern.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Workload:
    name: str
    dtype: str                      # "f32" | "f16" | "bf16"
    sources: dict                   # name -> storage array
    chain: list                     # statements, see module docstring
    consumer: dict                  # what reads the chain's results
    index_tables: dict = field(default_factory=dict)   # name -> int32 array
    note: str = ""


def encode(x32: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32 array to the storage type (round-to-nearest-even)."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "f32":
        return x32
    if dtype == "f16":
        return x32.astype(np.float16)
    if dtype == "bf16":
        out = np.empty(x32.shape, dtype=np.uint16)
        src, dst = x32.reshape(-1).view(np.uint32), out.reshape(-1)
        step = 1 << 22                         # in slices: the temporaries stay in cache
        for i in range(0, src.size, step):
            bits = src[i:i + step]
            t = (bits >> np.uint32(16)) & np.uint32(1)
            t += bits
            t += np.uint32(0x7FFF)
            t >>= np.uint32(16)
            dst[i:i + step] = t
        return out
    raise ValueError(dtype)


def _rng(seed: int, k: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, k]))


def _uniform(seed, k, shape, dtype):
    return encode(_rng(seed, k).uniform(-1.0, 1.0, size=shape).astype(np.float32), dtype)


def _normal(seed, k, shape, std, dtype):
    """N(0, std) in float32 from stream (seed, k), rounded to `dtype`.  Large tensors are drawn in
    slices from the one generator (the stream, and so every value, is that of a single draw)."""
    g = _rng(seed, k)
    n = int(np.prod(shape))
    step = 1 << 22
    if n <= step:
        x = g.standard_normal(size=shape, dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        return encode(x, dtype)
    out = np.empty(n, dtype={"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype])
    buf = np.empty(step, dtype=np.float32)
    for i in range(0, n, step):
        x = buf[:min(step, n - i)]
        g.standard_normal(out=x, dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        out[i:i + x.size] = encode(x, dtype)
    return out.reshape(shape)


# ----------------------------------------------------------------------------------------
# C1: tiny chain, fp32
# ----------------------------------------------------------------------------------------
def c1_tiny_chain(seed: int = 0, a: int = 4, b: int = 6, c: int = 8, lo: int = 4, hi: int = 20,
                  ny: int = 5) -> Workload:
    """X[a,b,c] -> permute(2,0,1) -> reshape[c, a*b] -> slice cols lo:hi -> concat with
    Y[c,ny] along dim 1 -> add Z -> row-sum.  Defaults are the benchmark's sizes."""
    w = hi - lo + ny
    src = {
        "X": _uniform(seed, 0, (a, b, c), "f32"),
        "Y": _uniform(seed, 1, (c, ny), "f32"),
        "Z": _uniform(seed, 2, (c, w), "f32"),
    }
    chain = [
        ("t1", "permute", ("X",), {"perm": (2, 0, 1)}),
        ("t2", "reshape", ("t1",), {"shape": (c, a * b)}),
        ("t3", "slice", ("t2",), {"dim": 1, "start": lo, "stop": hi, "step": 1}),
        ("V", "concat", ("t3", "Y"), {"dim": 1}),
    ]
    return Workload("c1_tiny_chain", "f32", src, chain,
                    {"kind": "add_rowsum", "x": "V", "y": "Z"})


def rowsum_chain_large(seed: int = 0, A: int = 32, B: int = 8192, C0: int = 128, ny: int = 1024) -> Workload:
    """Config 1's consumer at a memory-bound size, on a chain whose map keeps runs of C0 elements:
    X[A,B,C0] -> permute(1,0,2) -> reshape[B, A*C0] -> concat along dim 1 with Y[B,ny] -> add Z ->
    row-sum (fp32).  Defaults: 134 MB + 34 MB + 168 MB read per pass."""
    C = A * C0 + ny
    src = {
        "X": _normal(seed, 0, (A, B, C0), 1.0, "f32"),
        "Y": _normal(seed, 1, (B, ny), 1.0, "f32"),
        "Z": _normal(seed, 2, (B, C), 1.0, "f32"),
    }
    chain = [
        ("t1", "permute", ("X",), {"perm": (1, 0, 2)}),
        ("t2", "reshape", ("t1",), {"shape": (B, A * C0)}),
        ("V", "concat", ("t2", "Y"), {"dim": 1}),
    ]
    return Workload("rowsum_chain_large", "f32", src, chain, {"kind": "add_rowsum", "x": "V", "y": "Z"})


# ----------------------------------------------------------------------------------------
# C2: Llama-3-8B-shaped decode segment, bf16
# ----------------------------------------------------------------------------------------
def c2_chain(B: int, Hkv: int, G: int, S: int, D: int) -> list:
    """Statements of the decode segment (no data): Q, K, V as seen by the attention kernel."""
    Hq = Hkv * G
    sizes = (Hq * D, Hkv * D, Hkv * D)
    chain = [
        ("q0", "split", ("QKV",), {"dim": 2, "sizes": sizes, "output": 0}),
        ("q1", "reshape", ("q0",), {"shape": (B, 1, Hq, D)}),
        ("Q", "permute", ("q1",), {"perm": (0, 2, 1, 3)}),
    ]
    for nm, out_i, cache in (("k", 1, "Kcache"), ("v", 2, "Vcache")):
        chain += [
            (nm + "0", "split", ("QKV",), {"dim": 2, "sizes": sizes, "output": out_i}),
            (nm + "1", "reshape", (nm + "0",), {"shape": (B, 1, Hkv, D)}),
            (nm + "n", "permute", (nm + "1",), {"perm": (0, 2, 1, 3)}),
            (nm + "p", "slice", (cache,), {"dim": 2, "start": 0, "stop": S - 1, "step": 1}),
            (nm + "f", "concat", (nm + "p", nm + "n"), {"dim": 2}),
            (nm + "u", "unsqueeze", (nm + "f",), {"dim": 2}),
            (nm + "x", "expand", (nm + "u",), {"shape": (B, Hkv, G, S, D)}),
            (nm.upper(), "reshape", (nm + "x",), {"shape": (B, Hq, S, D)}),
        ]
    return chain


def c2_decode_attention(seed: int = 0, B: int = 8, Hkv: int = 8, G: int = 4, S: int = 4096,
                        D: int = 128, dtype: str = "bf16", poison_last_slot: bool = False) -> Workload:
    """Fused QKV output [B,1,(Hq+2Hkv)*D] is cut into Q, K_new, V_new; K_new/V_new take the
    last slot of a cache of capacity S (the first S-1 slots come from the cache); the Hkv
    heads are broadcast G-fold to the Hq = Hkv*G query heads; decode attention over S keys.
    ``poison_last_slot`` writes NaN into the cache slot the new token replaces: that slot
    must never be read."""
    Hq = Hkv * G
    E = (Hq + 2 * Hkv) * D
    qkv = _normal(seed, 0, (B, 1, E), 1.0, dtype)
    kc32 = _rng(seed, 1).standard_normal(size=(B, Hkv, S, D), dtype=np.float32)
    vc32 = _rng(seed, 2).standard_normal(size=(B, Hkv, S, D), dtype=np.float32)
    if poison_last_slot:
        kc32[:, :, S - 1, :] = np.nan
        vc32[:, :, S - 1, :] = np.nan
    src = {"QKV": qkv, "Kcache": encode(kc32, dtype), "Vcache": encode(vc32, dtype)}
    del kc32, vc32
    chain = c2_chain(B, Hkv, G, S, D)
    return Workload("c2_decode_attention", dtype, src, chain,
                    {"kind": "decode_attn", "q": "Q", "k": "K", "v": "V",
                     "scale": 1.0 / float(np.sqrt(D))})


# ----------------------------------------------------------------------------------------
# C3: attention-output transpose into o-proj GEMM, bf16
# ----------------------------------------------------------------------------------------
def c3_oproj_gemm(seed: int = 0, B: int = 16, H: int = 32, S: int = 512, D: int = 128,
                  N: int = 4096, dtype: str = "bf16") -> Workload:
    src = {
        "O": _normal(seed, 0, (B, H, S, D), 1.0, dtype),
        "W": _normal(seed, 1, (H * D, N), 0.02, dtype),
    }
    chain = [
        ("o1", "permute", ("O",), {"perm": (0, 2, 1, 3)}),
        ("A", "reshape", ("o1",), {"shape": (B * S, H * D)}),
    ]
    return Workload("c3_oproj_gemm", dtype, src, chain, {"kind": "gemm", "a": "A", "b": "W"})


# ----------------------------------------------------------------------------------------
# C4: window partition -> LayerNorm -> linear, fp16
# ----------------------------------------------------------------------------------------
def c4_window_ln_linear(seed: int = 0, B: int = 32, R: int = 56, win: int = 7, C: int = 128,
                        N: int = 384, dtype: str = "f16") -> Workload:
    nw = R // win
    assert nw * win == R
    src = {
        "X": _normal(seed, 0, (B, R, R, C), 1.0, dtype),
        "W": _normal(seed, 1, (C, N), 0.02, dtype),
    }
    chain = [
        ("x1", "reshape", ("X",), {"shape": (B, nw, win, nw, win, C)}),
        ("x2", "permute", ("x1",), {"perm": (0, 1, 3, 2, 4, 5)}),
        ("T", "reshape", ("x2",), {"shape": (B * nw * nw, win * win, C)}),
    ]
    return Workload("c4_window_ln_linear", dtype, src, chain,
                    {"kind": "ln_linear", "x": "T", "w": "W", "eps": 1e-5})


# ----------------------------------------------------------------------------------------
# C5: MoE token dispatch, bf16
# ----------------------------------------------------------------------------------------
def c5_moe_dispatch(seed: int = 0, T: int = 16384, Hd: int = 4096, E: int = 8, N: int = 14336,
                    dtype: str = "bf16") -> Workload:
    """Every token goes to two distinct experts drawn uniformly; expert e reads its tokens
    (ascending token id) through an index table and multiplies them by its own weight."""
    src = {
        "tokens": _normal(seed, 0, (T, Hd), 1.0, dtype),
        "W": _normal(seed, 1, (E, Hd, N), 0.02, dtype),
    }
    g = _rng(seed, 2)
    first = g.integers(0, E, size=T)
    second = (first + 1 + g.integers(0, E - 1, size=T)) % E      # distinct from `first`
    tables = {}
    chain = []
    a_names, b_names = [], []
    for e in range(E):
        tok = np.nonzero((first == e) | (second == e))[0].astype(np.int32)   # ascending
        tables["idx%d" % e] = tok
        chain.append(("A%d" % e, "index_select", ("tokens",), {"dim": 0, "index": "idx%d" % e}))
        chain.append(("w%d" % e, "slice", ("W",), {"dim": 0, "start": e, "stop": e + 1, "step": 1}))
        chain.append(("B%d" % e, "reshape", ("w%d" % e,), {"shape": (Hd, N)}))
        a_names.append("A%d" % e)
        b_names.append("B%d" % e)
    return Workload("c5_moe_dispatch", dtype, src, chain,
                    {"kind": "grouped_gemm", "a": a_names, "b": b_names}, tables)


# ----------------------------------------------------------------------------------------
# QKV projection that writes through a virtual tensor (producer-side store), bf16
# ----------------------------------------------------------------------------------------
def qkv_store_chain(B: int, Hq: int, Hkv: int, cap: int, D: int, pos: int, T: int = 1):
    """The projection's output C[B*T, (Hq+2Hkv)*D] seen as a virtual tensor of three physical
    tensors (Fig. 4): columns [0, Hq*D) are the Q buffer, the next Hkv*D columns are slots
    pos .. pos+T-1 of the K cache [B,Hkv,cap,D], the last Hkv*D those of the V cache."""
    chain = [("q2", "reshape", ("Qbuf",), {"shape": (B * T, Hq * D)})]
    for n, cache in (("k", "Kcache"), ("v", "Vcache")):
        chain += [
            (n + "s", "slice", (cache,), {"dim": 2, "start": pos, "stop": pos + T}),      # [B,Hkv,T,D]
            (n + "p", "permute", (n + "s",), {"perm": (0, 2, 1, 3)}),                       # [B,T,Hkv,D]
            (n + "2", "reshape", (n + "p",), {"shape": (B * T, Hkv * D)}),
        ]
    chain.append(("Cout", "concat", ("q2", "k2", "v2"), {"dim": 1}))
    return chain


def qkv_proj_store(seed: int = 0, B: int = 8, hidden: int = 4096, Hq: int = 32, Hkv: int = 8, D: int = 128,
                   cap: int = 4096, pos: int = 4095, T: int = 1, dtype: str = "bf16") -> Workload:
    """Decode step (T = 1) or a chunk of T new tokens per sequence: X[B*T, hidden] . W[hidden, (Hq+2Hkv)*D],
    result stored straight into the Q buffer and the cache slots.  The caches and the Q buffer
    hold random values beforehand so that a store to a wrong place, or a missing one, shows."""
    E = (Hq + 2 * Hkv) * D
    src = {
        "X": _normal(seed, 0, (B * T, hidden), 1.0, dtype),
        "W": _normal(seed, 1, (hidden, E), 0.02, dtype),
        "Qbuf": _normal(seed, 2, (B, T, Hq * D), 1.0, dtype),
        "Kcache": _normal(seed, 3, (B, Hkv, cap, D), 1.0, dtype),
        "Vcache": _normal(seed, 4, (B, Hkv, cap, D), 1.0, dtype),
    }
    return Workload("qkv_proj_store", dtype, src, qkv_store_chain(B, Hq, Hkv, cap, D, pos, T),
                    {"kind": "gemm_store", "a": "X", "b": "W", "out": "Cout"})


def moe_combine(seed: int = 0, T: int = 16384, E: int = 8, N: int = 14336, dtype: str = "bf16") -> Workload:
    """The step after config 5: the expert outputs Y[2T, N] (expert-major, tokens ascending inside
    an expert, the layout config 5 writes) are read back per token and mixed with the two routing
    weights.  Routing as in config 5 (two distinct experts per token, uniform); weights = softmax
    of two N(0,1) logits, fp32."""
    g = _rng(seed, 2)
    first = g.integers(0, E, size=T)
    second = (first + 1 + g.integers(0, E - 1, size=T)) % E
    lo, hi = np.minimum(first, second), np.maximum(first, second)
    counts = np.bincount(np.concatenate([first, second]), minlength=E)
    offset = np.concatenate([[0], np.cumsum(counts)[:-1]])
    rank = np.zeros((E, T), dtype=np.int64)                  # rank[e, t] = tokens < t routed to e
    for e in range(E):
        routed = ((first == e) | (second == e)).astype(np.int64)
        rank[e] = np.cumsum(routed) - routed
    t = np.arange(T)
    pos0 = (offset[lo] + rank[lo, t]).astype(np.int32)
    pos1 = (offset[hi] + rank[hi, t]).astype(np.int32)
    logits = _rng(seed, 3).standard_normal(size=(T, 2)).astype(np.float32)
    ex = np.exp(logits - logits.max(axis=1, keepdims=True))
    weights = (ex / ex.sum(axis=1, keepdims=True)).astype(np.float32)
    src = {"Y": _normal(seed, 0, (2 * T, N), 1.0, dtype)}
    chain = [("x", "index_select", ("Y",), {"dim": 0, "index": "pos0"}),
             ("y", "index_select", ("Y",), {"dim": 0, "index": "pos1"})]
    return Workload("moe_combine", dtype, src, chain,
                    {"kind": "weighted_sum", "x": "x", "y": "y", "weights": weights},
                    {"pos0": pos0, "pos1": pos1})


def paged_decode_attention(seed: int = 0, B: int = 8, Hkv: int = 8, G: int = 4, pages_per_seq: int = 32,
                           page: int = 128, D: int = 128, pool_pages: int = 0, dtype: str = "bf16",
                           poison_unused: bool = False) -> Workload:
    """Decode attention over a paged KV cache: K and V live in pools [pool_pages, Hkv, page, D] and
    sequence b owns the pages bt[b*P .. b*P+P) (distinct, in random order).  The chain gathers the
    pages (index_select), puts them in context order and broadcasts the kv heads, as a framework
    without paged kernels would; ``poison_unused`` fills the pages no sequence owns with NaN."""
    Hq, P = Hkv * G, pages_per_seq
    S = P * page
    NP = pool_pages or (B * P + 3)
    assert NP >= B * P
    bt = _rng(seed, 5).permutation(NP)[:B * P].astype(np.int32)
    pools = {}
    for k, name in ((1, "Kpool"), (2, "Vpool")):
        x = _rng(seed, k).standard_normal(size=(NP, Hkv, page, D), dtype=np.float32)
        if poison_unused:
            unused = np.setdiff1d(np.arange(NP), bt)
            x[unused] = np.nan
        pools[name] = encode(x, dtype)
        del x
    src = {"Qs": _normal(seed, 0, (B, 1, Hq * D), 1.0, dtype), **pools}
    chain = [("q1", "reshape", ("Qs",), {"shape": (B, 1, Hq, D)}),
             ("Q", "permute", ("q1",), {"perm": (0, 2, 1, 3)})]
    for nm, pool in (("k", "Kpool"), ("v", "Vpool")):
        chain += [
            (nm + "g", "index_select", (pool,), {"dim": 0, "index": "bt"}),                 # [B*P, Hkv, page, D]
            (nm + "r", "reshape", (nm + "g",), {"shape": (B, P, Hkv, page, D)}),
            (nm + "t", "permute", (nm + "r",), {"perm": (0, 2, 1, 3, 4)}),                    # [B, Hkv, P, page, D]
            (nm + "c", "reshape", (nm + "t",), {"shape": (B, Hkv, S, D)}),
            (nm + "u", "unsqueeze", (nm + "c",), {"dim": 2}),
            (nm + "x", "expand", (nm + "u",), {"shape": (B, Hkv, G, S, D)}),
            (nm.upper(), "reshape", (nm + "x",), {"shape": (B, Hq, S, D)}),
        ]
    return Workload("paged_decode_attention", dtype, src, chain,
                    {"kind": "decode_attn", "q": "Q", "k": "K", "v": "V", "scale": 1.0 / float(np.sqrt(D))},
                    index_tables={"bt": bt})


def decode_segment(seed: int = 0, B: int = 8, hidden: int = 4096, Hkv: int = 8, G: int = 4, D: int = 128,
                   cap: int = 4096, pos: int = 4095, dtype: str = "bf16"):
    """The paper's motivating example end to end (Sec. 3.1): the merged QKV projection stores Q
    and the new K, V rows through a virtual tensor (stage 1), then decode attention reads the Q
    buffer and slots 0..pos of the un-expanded caches (stage 2).  Returns the two workloads; they
    name the same Qbuf / Kcache / Vcache, stage 2 sees what stage 1 stored."""
    Hq = Hkv * G
    S = pos + 1
    st1 = qkv_proj_store(seed, B, hidden, Hq, Hkv, D, cap, pos, 1, dtype)
    chain = [("q1", "reshape", ("Qbuf",), {"shape": (B, 1, Hq, D)}),
             ("Q", "permute", ("q1",), {"perm": (0, 2, 1, 3)})]
    for nm, cache in (("k", "Kcache"), ("v", "Vcache")):
        chain += [
            (nm + "s", "slice", (cache,), {"dim": 2, "start": 0, "stop": S, "step": 1}),
            (nm + "u", "unsqueeze", (nm + "s",), {"dim": 2}),
            (nm + "x", "expand", (nm + "u",), {"shape": (B, Hkv, G, S, D)}),
            (nm.upper(), "reshape", (nm + "x",), {"shape": (B, Hq, S, D)}),
        ]
    src2 = {k: st1.sources[k] for k in ("Qbuf", "Kcache", "Vcache")}
    st2 = Workload("decode_segment_attention", dtype, src2, chain,
                   {"kind": "decode_attn", "q": "Q", "k": "K", "v": "V", "scale": 1.0 / float(np.sqrt(D))})
    return st1, st2


CONFIGS = {
    "c1": c1_tiny_chain,
    "c2": c2_decode_attention,
    "c3": c3_oproj_gemm,
    "c4": c4_window_ln_linear,
    "c5": c5_moe_dispatch,
    "rowsum_large": rowsum_chain_large,
    "qkv_store": qkv_proj_store,
    "paged": paged_decode_attention,
    "moe_combine": moe_combine,
}


# ----------------------------------------------------------------------------------------
# Random chains for property tests (valid by construction; small extents)
# ----------------------------------------------------------------------------------------
def _factorizations(n: int, g: np.random.Generator, max_dims: int = 4):
    """A random ordered factorization of n into 1..max_dims factors."""
    dims = []
    rest = n
    for _ in range(int(g.integers(1, max_dims + 1)) - 1):
        divs = [d for d in range(1, rest + 1) if rest % d == 0]
        d = int(divs[int(g.integers(0, len(divs)))])
        dims.append(d)
        rest //= d
    dims.append(rest)
    g.shuffle(dims)
    return tuple(int(d) for d in dims)


def random_chain(seed: int, n_ops: int = 5, max_extent: int = 6, dtype: str = "f32",
                 ops=("permute", "reshape", "slice", "split", "concat", "unsqueeze", "expand",
                      "index_select")) -> Workload:
    """A random valid chain over small float sources filled with distinct integers (so that a
    value identifies the element it came from).  The result value is named "R"."""
    g = _rng(seed, 1000)
    counter = [0]
    sources, tables, chain = {}, {}, []

    def new_source(shape):
        name = "S%d" % len(sources)
        n = int(np.prod(shape)) if len(shape) else 1
        vals = np.arange(counter[0], counter[0] + n, dtype=np.float32).reshape(shape)
        counter[0] += n
        sources[name] = encode(vals, dtype)
        return name

    nd = int(g.integers(1, 5))
    shape = tuple(int(g.integers(1, max_extent + 1)) for _ in range(nd))
    cur = new_source(shape)
    k = 0
    while k < n_ops:
        op = ops[int(g.integers(0, len(ops)))]
        out = "v%d" % k
        nd = len(shape)
        if op == "permute":
            perm = tuple(int(p) for p in g.permutation(nd))
            chain.append((out, "permute", (cur,), {"perm": perm}))
            shape = tuple(shape[p] for p in perm)
        elif op == "reshape":
            n = int(np.prod(shape))
            new = _factorizations(n, g)
            chain.append((out, "reshape", (cur,), {"shape": new}))
            shape = new
        elif op == "slice":
            d = int(g.integers(0, nd))
            if shape[d] < 1:
                continue
            start = int(g.integers(0, shape[d]))
            stop = int(g.integers(start + 1, shape[d] + 1))
            step = int(g.integers(1, 3))
            chain.append((out, "slice", (cur,), {"dim": d, "start": start, "stop": stop, "step": step}))
            shape = shape[:d] + ((stop - start + step - 1) // step,) + shape[d + 1:]
        elif op == "split":
            d = int(g.integers(0, nd))
            if shape[d] < 2:
                continue
            cut = int(g.integers(1, shape[d]))
            sizes = (cut, shape[d] - cut)
            which = int(g.integers(0, 2))
            chain.append((out, "split", (cur,), {"dim": d, "sizes": sizes, "output": which}))
            shape = shape[:d] + (sizes[which],) + shape[d + 1:]
        elif op == "concat":
            d = int(g.integers(0, nd))
            ext = int(g.integers(1, max_extent + 1))
            oshape = shape[:d] + (ext,) + shape[d + 1:]
            other = new_source(oshape)
            ins = (cur, other) if int(g.integers(0, 2)) == 0 else (other, cur)
            chain.append((out, "concat", ins, {"dim": d}))
            shape = shape[:d] + (shape[d] + ext,) + shape[d + 1:]
        elif op == "unsqueeze":
            if nd >= 6:
                continue
            d = int(g.integers(0, nd + 1))
            chain.append((out, "unsqueeze", (cur,), {"dim": d}))
            shape = shape[:d] + (1,) + shape[d:]
        elif op == "expand":
            ones = [i for i, s in enumerate(shape) if s == 1]
            if not ones:
                continue
            d = ones[int(g.integers(0, len(ones)))]
            new = shape[:d] + (int(g.integers(2, 5)),) + shape[d + 1:]
            chain.append((out, "expand", (cur,), {"shape": new}))
            shape = new
        elif op == "index_select":
            d = int(g.integers(0, nd))
            n_idx = int(g.integers(1, 8))
            tname = "idx%d" % len(tables)
            tables[tname] = g.integers(0, shape[d], size=n_idx).astype(np.int32)
            chain.append((out, "index_select", (cur,), {"dim": d, "index": tname}))
            shape = shape[:d] + (n_idx,) + shape[d + 1:]
        else:
            raise ValueError(op)
        cur = out
        k += 1
        if int(np.prod(shape)) > 4096:      # keep brute force cheap
            break
    chain.append(("R", "reshape", (cur,), {"shape": shape}))
    return Workload("random_chain_%d" % seed, dtype, sources, chain,
                    {"kind": "materialize", "x": "R"}, tables)
