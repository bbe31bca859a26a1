"""Consumers that read the dense result of a chain.  float64 throughout, except where a
reading of the paper's silence fixes the precision (stated at each function).
"""
from __future__ import annotations

import numpy as np


def decode(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored bits -> float64 values (exact)."""
    if dtype == "f32":
        assert x.dtype == np.float32
        return x.astype(np.float64)
    if dtype == "f16":
        assert x.dtype == np.float16
        return x.astype(np.float64)
    if dtype == "bf16":
        assert x.dtype == np.uint16
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def add_rowsum_f32(v: np.ndarray, z: np.ndarray) -> np.ndarray:
    """out[r] = sum_c (v[r,c] + z[r,c]) in float32.

    The benchmark asks for a bit-exact fp32 result and the paper fixes no summation order
    (its method only changes stage 1 and 3 of a kernel, Sec. 4.2).  Reading used here, the
    natural order of a 64-wide machine: the add is done first, in float32; partial sum l of
    64 takes the columns c = l, l+64, l+128, ... in ascending order starting from +0; the 64
    partial sums are then combined by the butterfly p[l] += p[l xor s] for s = 32, 16, 8, 4,
    2, 1 and the result is p[0].  Every operation is an IEEE float32 add (numpy float32
    arithmetic, no fused multiply-add is involved).
    """
    assert v.dtype == np.float32 and z.dtype == np.float32 and v.shape == z.shape and v.ndim == 2
    rows, cols = v.shape
    p = np.zeros((rows, 64), dtype=np.float32)
    for c in range(cols):
        t = v[:, c] + z[:, c]
        p[:, c % 64] = p[:, c % 64] + t
    lanes = np.arange(64)
    for s in (32, 16, 8, 4, 2, 1):
        p = p + p[:, lanes ^ s]
    return p[:, 0].copy()


def layernorm(x: np.ndarray, eps: float) -> np.ndarray:
    """Per-token LayerNorm over the last dim, gamma = 1, beta = 0, biased variance."""
    x = x.astype(np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def gemm(a: np.ndarray, w: np.ndarray) -> np.ndarray:
    """C[m,n] = sum_k A[m,k] W[k,n] on float64 values."""
    return np.matmul(a.astype(np.float64), w.astype(np.float64))


def ln_linear(x: np.ndarray, w: np.ndarray, eps: float, store_dtype: str = "f16") -> np.ndarray:
    """LayerNorm, rounded to the storage type (the tensor that a 16-bit graph would hand to the
    linear layer and that the matrix units consume), then the linear layer without bias.  The
    rounding is the one every 16-bit output takes: round_to below."""
    y = layernorm(x, eps)
    if store_dtype in ("f16", "bf16"):
        y = decode(round_to(y, store_dtype), store_dtype)
    lead = y.shape[:-1]
    out = gemm(y.reshape(-1, y.shape[-1]), w)
    return out.reshape(lead + (w.shape[1],))


def decode_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float):
    """q [B,H,1,D], k and v [B,H,S,D] (already expanded to the query heads) ->
    out [B,H,D] and the log-sum-exp of the scaled scores [B,H]."""
    B, H, one, D = q.shape
    assert one == 1 and k.shape == v.shape and k.shape[:2] == (B, H) and k.shape[3] == D
    out = np.empty((B, H, D), dtype=np.float64)
    lse = np.empty((B, H), dtype=np.float64)
    for b in range(B):
        qb = q[b, :, 0, :].astype(np.float64)                # [H,D]
        kb = k[b].astype(np.float64)                         # [H,S,D]
        vb = v[b].astype(np.float64)
        s = scale * np.einsum("hd,htd->ht", qb, kb)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        den = e.sum(axis=1, keepdims=True)
        out[b] = np.einsum("ht,htd->hd", e / den, vb)
        lse[b] = (m + np.log(den))[:, 0]
    return out, lse


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """float64 values -> stored bits of the 16-bit type, round to nearest even (the output type of
    a GEMM is the type of its inputs).  bf16 is rounded from the float32 nearest to the value."""
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        b = x.astype(np.float32).view(np.uint32)
        keep = b >> np.uint32(16)
        rest = b & np.uint32(0xFFFF)
        up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & np.uint32(1)) == 1))
        nan = (b & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        r = np.where(nan, keep | np.uint32(0x40), keep + up.astype(np.uint32))
        return r.astype(np.uint16)
    raise ValueError(dtype)


def weighted_sum(x: np.ndarray, y: np.ndarray, w: np.ndarray) -> np.ndarray:
    """out[r, :] = w[r, 0] x[r, :] + w[r, 1] y[r, :] in float64 (the combine of a mixture of
    experts: x, y the two expert outputs of token r, w its routing weights)."""
    w = w.astype(np.float64)
    return w[:, 0:1] * x + w[:, 1:2] * y
