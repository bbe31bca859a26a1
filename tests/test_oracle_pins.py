"""Pins for the CPU oracle (no GPU).  Each test checks the oracle against something other
than itself: brute-force index enumeration, algebraic invariants, closed forms the paper
prints or that follow by hand from the operator definitions, and textbook special cases."""
import itertools
import json
import os

import numpy as np
import pytest

import workloads
from oracle import consumers, dm_ops, index_maps
from oracle.run import run_workload

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_pins.json")))


def arange(shape, dtype=np.float32):
    return np.arange(int(np.prod(shape)), dtype=dtype).reshape(shape)


# ------------------------------------------------------------------ per-operator: brute force
CASES = [
    ("permute", [(2, 3, 4)], {"perm": (2, 0, 1)}),
    ("permute", [(2, 3, 4)], {"perm": (1, 2, 0)}),
    ("permute", [(3, 5)], {"perm": (1, 0)}),
    ("permute", [(2, 3, 2, 3)], {"perm": (0, 2, 1, 3)}),
    ("reshape", [(2, 3, 4)], {"shape": (6, 4)}),
    ("reshape", [(2, 3, 4)], {"shape": (4, 6)}),
    ("reshape", [(12,)], {"shape": (2, 2, 3)}),
    ("slice", [(5, 6)], {"dim": 1, "start": 1, "stop": 5, "step": 1}),
    ("slice", [(5, 6)], {"dim": 0, "start": 1, "stop": 5, "step": 2}),
    ("slice", [(7,)], {"dim": 0, "start": 2, "stop": 7, "step": 3}),
    ("split", [(4, 6)], {"dim": 1, "sizes": (1, 2, 3), "output": 0}),
    ("split", [(4, 6)], {"dim": 1, "sizes": (1, 2, 3), "output": 1}),
    ("split", [(4, 6)], {"dim": 1, "sizes": (1, 2, 3), "output": 2}),
    ("split", [(4, 6)], {"dim": 0, "sizes": (3, 1), "output": 1}),
    ("concat", [(2, 3), (2, 1), (2, 4)], {"dim": 1}),
    ("concat", [(2, 3), (5, 3)], {"dim": 0}),
    ("unsqueeze", [(2, 3)], {"dim": 0}),
    ("unsqueeze", [(2, 3)], {"dim": 1}),
    ("unsqueeze", [(2, 3)], {"dim": 2}),
    ("expand", [(2, 1, 3)], {"shape": (2, 4, 3)}),
    ("expand", [(1, 3, 1)], {"shape": (2, 3, 5)}),
    ("index_select", [(4, 3)], {"dim": 0, "index": "t"}),
    ("index_select", [(4, 3)], {"dim": 1, "index": "u"}),
]
TABLES = {"t": np.array([3, 0, 0, 2, 1, 3], np.int32), "u": np.array([2, 2, 0], np.int32)}


@pytest.mark.parametrize("op,shapes,p", CASES)
def test_dense_op_equals_bruteforce_definition(op, shapes, p):
    ins, base = [], 0
    for s in shapes:
        ins.append(arange(s) + base)
        base += 1000
    dense = dm_ops.run_statement(op, ins, p, TABLES)
    brute = index_maps.materialize_bruteforce(op, ins, p, TABLES)
    assert dense.shape == brute.shape
    assert dense.flags["C_CONTIGUOUS"]
    np.testing.assert_array_equal(dense, brute)


@pytest.mark.parametrize("seed", range(60))
def test_random_chain_dense_equals_pull_back(seed):
    wl = workloads.random_chain(seed, n_ops=6)
    env = dm_ops.run_chain(wl.chain, wl.sources, wl.index_tables)
    ch = index_maps.Chain(wl.chain, {k: v.shape for k, v in wl.sources.items()}, wl.index_tables)
    ref = ch.materialize_by_pull_back("R", wl.sources)
    np.testing.assert_array_equal(env["R"], ref)


# ------------------------------------------------------------------ invariants
def test_permute_inverse_is_identity_and_2d_is_textbook_transpose():
    x = arange((2, 3, 4, 5))
    for perm in itertools.permutations(range(4)):
        inv = tuple(int(i) for i in np.argsort(perm))
        np.testing.assert_array_equal(dm_ops.permute(dm_ops.permute(x, perm), inv), x)
    m = arange((3, 5))
    t = dm_ops.permute(m, (1, 0))
    for i in range(5):
        for j in range(3):
            assert t[i, j] == m[j, i]


def test_permute_convention_is_onnx():
    # out.shape[i] = in.shape[perm[i]]: [4,6,8] with perm (2,0,1) gives [8,4,6]
    x = arange((4, 6, 8))
    y = dm_ops.permute(x, (2, 0, 1))
    assert y.shape == (8, 4, 6)
    assert y[5, 3, 2] == x[3, 2, 5]
    # the inverse convention would give [6,8,4]: make sure that is NOT what we compute
    assert y.shape != (6, 8, 4)


def test_reshape_preserves_row_major_order():
    x = dm_ops.permute(arange((3, 4, 5)), (1, 0, 2))        # a dense array with shuffled values
    for shp in [(60,), (12, 5), (5, 12), (2, 6, 5), (2, 2, 3, 5)]:
        np.testing.assert_array_equal(dm_ops.reshape(x, shp).ravel(), x.ravel())


def test_stride_example_from_paper():
    # Sec. 2.1: shape (a,b,c) -> strides (bc, c, 1); offset of (i,j,k) = i*bc + j*c + k
    assert GOLD["stride_example"]["stride"] == ["b*c", "c", "1"]
    a, b, c = 3, 4, 5
    x = arange((a, b, c))
    flat = dm_ops.reshape(x, (a * b * c,))
    for i, j, k in itertools.product(range(a), range(b), range(c)):
        assert flat[i * b * c + j * c + k] == x[i, j, k]


def test_concat_split_roundtrip_and_slice_partition():
    x = arange((4, 7, 3))
    for dim, sizes in [(0, (1, 3)), (1, (2, 4, 1)), (2, (1, 1, 1))]:
        parts = dm_ops.split(x, dim, sizes)
        np.testing.assert_array_equal(dm_ops.concat(parts, dim), x)
        again = dm_ops.split(dm_ops.concat(parts, dim), dim, sizes)
        for p, q in zip(parts, again):
            np.testing.assert_array_equal(p, q)
    np.testing.assert_array_equal(dm_ops.slice_(x, 1, 0, 7, 1), x)
    even, odd = dm_ops.slice_(x, 1, 0, 7, 2), dm_ops.slice_(x, 1, 1, 7, 2)
    assert even.shape[1] == 4 and odd.shape[1] == 3
    np.testing.assert_array_equal(even[:, 2], x[:, 4])
    np.testing.assert_array_equal(odd[:, 2], x[:, 5])


def test_expand_closed_form_eq2():
    # Eq. 2: (a,b,c) -> (a,3b,c): offset = i*bc + (j%b)*c + k = i*bc + j*c + k - floor(j/b)*bc
    rep = GOLD["expand_closed_form"]["repeat"]
    a, b, c = 2, 3, 4
    x = arange((a, b, c))
    flat = x.ravel()
    u = dm_ops.unsqueeze(x, 1)                                # (a,1,b,c)
    e = dm_ops.expand(u, (a, rep, b, c))
    y = dm_ops.reshape(e, (a, rep * b, c))
    for i, j, k in itertools.product(range(a), range(rep * b), range(c)):
        off = i * b * c + j * c + k - (j // b) * b * c
        assert off == i * b * c + (j % b) * c + k
        assert y[i, j, k] == flat[off]
    # every replica equals the input; the first slice of an expanded dim is the input
    for r in range(rep):
        np.testing.assert_array_equal(e[:, r], x)
    np.testing.assert_array_equal(dm_ops.slice_(e, 1, 0, 1, 1), u)


def test_gqa_expand_repeat_index_inner():
    # query head h uses kv head h // G  (Sec. 3.1: Unsqueeze + Expand align KV heads to Q heads)
    G = GOLD["expand_ratio_llama3_8b"]["ratio"]
    kv = arange((2, 3, 5, 4))                                 # [B,Hkv,S,D]
    e = dm_ops.reshape(dm_ops.expand(dm_ops.unsqueeze(kv, 2), (2, 3, G, 5, 4)), (2, 3 * G, 5, 4))
    for h in range(3 * G):
        np.testing.assert_array_equal(e[:, h], kv[:, h // G])


def test_index_select_special_cases():
    x = arange((5, 3))
    np.testing.assert_array_equal(dm_ops.index_select(x, 0, np.arange(5)), x)
    perm = np.array([3, 0, 4, 1, 2])
    inv = np.argsort(perm)
    np.testing.assert_array_equal(dm_ops.index_select(dm_ops.index_select(x, 0, perm), 0, inv), x)
    y = dm_ops.index_select(x, 1, [2, 2, 0])
    for r in range(5):
        assert list(y[r]) == [x[r, 2], x[r, 2], x[r, 0]]


# ------------------------------------------------------------------ composed maps of the benchmark chains
def test_c1_closed_form():
    wl = workloads.c1_tiny_chain()
    env = dm_ops.run_chain(wl.chain, wl.sources)
    V, X, Y = env["V"], wl.sources["X"], wl.sources["Y"]
    assert V.shape == (8, 21)
    xf = X.ravel()
    for r in range(8):
        for c in range(21):
            if c < 16:
                cc = c + 4
                j, k = cc // 6, cc % 6
                assert V[r, c] == xf[48 * j + 8 * k + r] == X[j, k, r]
            else:
                assert V[r, c] == Y[r, c - 16]


def test_c2_closed_form_and_fig3_boundaries():
    B, Hkv, G, S, D = 2, 8, 4, 6, 128
    wl = workloads.c2_decode_attention(B=B, Hkv=Hkv, G=G, S=S, D=D)
    bounds = GOLD["fig3_qkv_columns"]["boundaries"]
    assert wl.sources["QKV"].shape == (B, 1, bounds[2])
    ch = index_maps.Chain(wl.chain, {k: v.shape for k, v in wl.sources.items()})
    env = dm_ops.run_chain(wl.chain, wl.sources)
    Hq = Hkv * G
    assert env["K"].shape == (B, Hq, S, D) and env["Q"].shape == (B, Hq, 1, D)
    rng = np.random.default_rng(0)
    for _ in range(400):
        b, h, t, d = (int(rng.integers(0, n)) for n in (B, Hq, S, D))
        for name, cache, col0 in (("K", "Kcache", bounds[0]), ("V", "Vcache", bounds[1])):
            src, y = ch.pull_back(name, (b, h, t, d))
            if t < S - 1:
                assert (src, y) == (cache, (b, h // G, t, d))
                assert env[name][b, h, t, d] == wl.sources[cache][b, h // G, t, d]
            else:
                assert (src, y) == ("QKV", (b, 0, col0 + (h // G) * D + d))
                assert env[name][b, h, t, d] == wl.sources["QKV"][b, 0, col0 + (h // G) * D + d]
        src, y = ch.pull_back("Q", (b, h, 0, d))
        assert (src, y) == ("QKV", (b, 0, h * D + d)) and y[2] < bounds[0]


def test_c3_closed_form():
    B, H, S, D = 2, 3, 5, 4
    wl = workloads.c3_oproj_gemm(B=B, H=H, S=S, D=D, N=8)
    env = dm_ops.run_chain(wl.chain, wl.sources)
    A, O = env["A"], wl.sources["O"]
    assert A.shape == (B * S, H * D)
    of = O.ravel()
    for m in range(B * S):
        for k in range(H * D):
            assert A[m, k] == O[m // S, k // D, m % S, k % D]
            assert A[m, k] == of[(m // S) * H * S * D + (k // D) * S * D + (m % S) * D + k % D]


def test_c4_closed_form():
    B, R, win, C = 2, 6, 3, 4
    wl = workloads.c4_window_ln_linear(B=B, R=R, win=win, C=C, N=8)
    env = dm_ops.run_chain(wl.chain, wl.sources)
    T, X = env["T"], wl.sources["X"]
    nw = R // win
    assert T.shape == (B * nw * nw, win * win, C)
    for w in range(B * nw * nw):
        b, wh, ww = w // (nw * nw), (w // nw) % nw, w % nw
        for p in range(win * win):
            ih, iw = p // win, p % win
            np.testing.assert_array_equal(T[w, p], X[b, wh * win + ih, ww * win + iw])


def test_c5_routing_structure():
    wl = workloads.c5_moe_dispatch(T=500, Hd=8, E=8, N=4)
    count = np.zeros(500, int)
    total = 0
    for e in range(8):
        idx = wl.index_tables["idx%d" % e]
        assert idx.dtype == np.int32
        assert np.all(np.diff(idx) > 0)                      # strictly ascending => distinct
        count[idx] += 1
        total += len(idx)
    assert total == 2 * 500 and np.all(count == 2)
    env = dm_ops.run_chain(wl.chain, wl.sources, wl.index_tables)
    for e in range(8):
        idx = wl.index_tables["idx%d" % e]
        for r, tkn in enumerate(idx):
            np.testing.assert_array_equal(env["A%d" % e][r], wl.sources["tokens"][tkn])
        np.testing.assert_array_equal(env["B%d" % e], wl.sources["W"][e])


# ------------------------------------------------------------------ consumers
def test_add_rowsum_order_and_exactness():
    # dyadic values: every order gives the same float32 sum
    rng = np.random.default_rng(1)
    v = (rng.integers(-64, 64, size=(5, 200)) / 8.0).astype(np.float32)
    z = (rng.integers(-64, 64, size=(5, 200)) / 8.0).astype(np.float32)
    out = consumers.add_rowsum_f32(v, z)
    np.testing.assert_array_equal(out, (v.astype(np.float64) + z).sum(axis=1).astype(np.float32))
    # order pin: lanes 0 and 2 cancel first (butterfly step 2), lane 1 joins last
    v = np.array([[1e8, 1.0, -1e8]], np.float32)
    assert consumers.add_rowsum_f32(v, np.zeros_like(v))[0] == np.float32(1.0)
    assert (np.float32(1e8) + np.float32(1.0)) + np.float32(-1e8) == np.float32(0.0)   # sequential differs
    # column 64 goes to lane 0 after column 0: (1e8 + -1e8) + ... exact 2.0 only in that order
    v = np.zeros((1, 66), np.float32)
    v[0, 0], v[0, 64], v[0, 1], v[0, 65] = 1e8, -1e8, 1.0, 1.0
    assert consumers.add_rowsum_f32(v, np.zeros_like(v))[0] == np.float32(2.0)
    # general inputs: within 1e-5 of the float64 sum
    wl = workloads.c1_tiny_chain()
    res = run_workload(wl)
    assert res["out"].dtype == np.float32 and res["out"].shape == (8,)
    assert np.max(np.abs(res["out"].astype(np.float64) - res["out_f64"])) <= 1e-5


def test_layernorm_properties():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(7, 128)) * 3 + 1.5
    eps = 1e-5
    y = consumers.layernorm(x, eps)
    assert np.max(np.abs(y.mean(axis=1))) < 1e-12
    var = x.var(axis=1)
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(consumers.layernorm(x + 10.0, eps), y, atol=1e-9)
    np.testing.assert_array_equal(consumers.layernorm(np.full((2, 128), 3.25), eps), np.zeros((2, 128)))
    # hand value: row [1,3] -> mean 2, var 1 -> (-1, 1)/sqrt(1+eps)
    np.testing.assert_allclose(consumers.layernorm(np.array([[1.0, 3.0]]), eps),
                               np.array([[-1.0, 1.0]]) / np.sqrt(1 + eps), rtol=1e-15)


def test_gemm_special_cases():
    rng = np.random.default_rng(3)
    a = rng.normal(size=(5, 7))
    w = rng.normal(size=(7, 4))
    np.testing.assert_array_equal(consumers.gemm(a, np.eye(7)), a)
    onehot = np.zeros((3, 7))
    onehot[0, 2] = onehot[1, 6] = onehot[2, 0] = 1
    np.testing.assert_array_equal(consumers.gemm(onehot, w), w[[2, 6, 0]])
    ref = np.zeros((5, 4))
    for m in range(5):
        for n in range(4):
            for k in range(7):
                ref[m, n] += a[m, k] * w[k, n]
    np.testing.assert_allclose(consumers.gemm(a, w), ref, rtol=1e-13, atol=1e-13)
    # orientation: a non-square product cannot be confused with its transpose
    assert consumers.gemm(a, w).shape == (5, 4)
    np.testing.assert_allclose(consumers.gemm(2 * a, w) + consumers.gemm(a, w), 3 * consumers.gemm(a, w), rtol=1e-12)


def test_ln_linear_rounds_between_hand_case():
    """A row whose normalised values are known by hand, with weights that make the rounding
    between LayerNorm and the product visible.  Row [0,0,0,4]: mean 1, deviations [-1,-1,-1,3],
    biased variance 3, so y = [-1,-1,-1,3] / sqrt(3) = [-0.57735.., 1.73205..] (eps = 1e-5 moves
    them by 2e-6 relative, far from any rounding boundary).
      f16  (ulp 2^-11 below 1, 2^-10 above):  -1182/2048 = -0.5771484375,  1774/1024 = 1.732421875
      bf16 (ulp 2^-8 below 1, 2^-7 above):    -148/256   = -0.578125,      222/128   = 1.734375
    Column 0 of W picks y[0]; column 1 = 1024 * (sum of the row): 0 without rounding, and
    1024 * (1.732421875 - 3 * 0.5771484375) = 1.0 in f16, 1024 * (1.734375 - 3 * 0.578125) = 0 in bf16."""
    x = np.array([[0.0, 0.0, 0.0, 4.0]])
    w = np.array([[1.0, 1024.0], [0.0, 1024.0], [0.0, 1024.0], [0.0, 1024.0]])
    f16 = consumers.ln_linear(x, w, 1e-5, "f16")
    bf16 = consumers.ln_linear(x, w, 1e-5, "bf16")
    assert f16.tolist() == [[-0.5771484375, 1.0]]
    assert bf16.tolist() == [[-0.578125, 0.0]]
    # the unrounded product differs from both in column 0 and is (nearly) 0 in column 1
    plain = consumers.gemm(consumers.layernorm(x, 1e-5), w)
    assert abs(plain[0, 0] + 0.5773493) < 1e-6 and abs(plain[0, 1]) < 1e-9
    # leading dims are kept: [2,1,4] -> [2,1,2]
    assert consumers.ln_linear(np.stack([x, 2 * x]), w, 1e-5, "bf16").shape == (2, 1, 2)


def test_ln_linear_rounding_is_round_to_nearest_even_on_ties():
    """Values that sit exactly between two bf16 / f16 numbers after LayerNorm cannot be made by
    hand (the normalisation is irrational), so ties are checked on the rounding itself, which
    ln_linear shares with every 16-bit output: 1 + 2^-8 -> 1 (even), 1 + 3 * 2^-8 -> 1 + 2^-6."""
    v = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -20])
    got = consumers.decode(consumers.round_to(v, "bf16"), "bf16")
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, -1.0, 1.0 + 2.0 ** -7]


def test_grouped_gemm_rows_are_expert_major():
    """Config 5's output buffer: expert 0's rows first (its tokens in ascending id), then expert
    1's, ...; row r of expert e's block is tokens[idx_e[r]] . W[e].  Checked on a tiny case with
    plain loops over the routing tables, values chosen so that every product is exact."""
    wl = workloads.c5_moe_dispatch(seed=7, T=12, Hd=4, E=3, N=5)
    rng = np.random.default_rng(0)
    tok = rng.integers(-3, 4, size=(12, 4)).astype(np.float32)
    W = rng.integers(-2, 3, size=(3, 4, 5)).astype(np.float32)
    wl.sources["tokens"], wl.sources["W"] = workloads.encode(tok, "bf16"), workloads.encode(W, "bf16")
    out = run_workload(wl)["out"]
    assert out.shape == (24, 5)
    r = 0
    for e in range(3):
        idx = wl.index_tables["idx%d" % e]
        assert list(idx) == sorted(set(idx))
        for t in idx:
            want = [sum(float(tok[t, k]) * float(W[e, k, n]) for k in range(4)) for n in range(5)]
            assert out[r].tolist() == want, (e, t, r)
            r += 1
    assert r == 24


def _naive_attention(q, k, v, scale):
    B, H, _, D = q.shape
    S = k.shape[2]
    out = np.zeros((B, H, D))
    for b in range(B):
        for h in range(H):
            s = [scale * sum(q[b, h, 0, d] * k[b, h, t, d] for d in range(D)) for t in range(S)]
            m = max(s)
            e = [np.exp(si - m) for si in s]
            den = sum(e)
            for t in range(S):
                for d in range(D):
                    out[b, h, d] += e[t] / den * v[b, h, t, d]
    return out


def test_decode_attention_special_cases():
    rng = np.random.default_rng(5)
    B, H, S, D = 2, 3, 9, 4
    q = rng.normal(size=(B, H, 1, D))
    k = rng.normal(size=(B, H, S, D))
    v = rng.normal(size=(B, H, S, D))
    out, lse = consumers.decode_attention(q, k, v, 0.5)
    np.testing.assert_allclose(out, _naive_attention(q, k, v, 0.5), rtol=1e-12, atol=1e-12)
    # all keys equal -> uniform weights -> mean of V
    k_same = np.broadcast_to(k[:, :, :1], k.shape)
    out2, lse2 = consumers.decode_attention(q, k_same, v, 0.5)
    np.testing.assert_allclose(out2, v.mean(axis=2), rtol=1e-12)
    s0 = 0.5 * np.einsum("bhd,bhd->bh", q[:, :, 0], k[:, :, 0])
    np.testing.assert_allclose(lse2, s0 + np.log(S), rtol=1e-12)
    # one key with a huge logit -> that V row
    k_big = k.copy()
    k_big[:, :, 4] = 1000.0 * q[:, :, 0]
    out3, _ = consumers.decode_attention(q, k_big, v, 0.5)
    np.testing.assert_allclose(out3, v[:, :, 4], rtol=1e-9, atol=1e-9)
    # permuting (key, value) pairs along the context changes nothing
    perm = rng.permutation(S)
    out4, lse4 = consumers.decode_attention(q, k[:, :, perm], v[:, :, perm], 0.5)
    np.testing.assert_allclose(out4, out, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lse4, lse, rtol=1e-12)
    # scale matters (a dropped scale fails here)
    out5, _ = consumers.decode_attention(q, k, v, 1.0)
    assert np.max(np.abs(out5 - out)) > 1e-3


def test_c2_workload_end_to_end_small():
    wl = workloads.c2_decode_attention(B=2, Hkv=2, G=4, S=33, D=128)
    res = run_workload(wl, keep_intermediates=True)
    env = res["env"]
    assert res["out"].shape == (2, 8, 128)
    # GQA: the four query heads of a group see identical K and V
    for h in range(8):
        np.testing.assert_array_equal(env["K"][:, h], env["K"][:, (h // 4) * 4])
    # the cache slot that the new token replaces must not matter
    wl_p = workloads.c2_decode_attention(B=2, Hkv=2, G=4, S=33, D=128, poison_last_slot=True)
    res_p = run_workload(wl_p)
    assert np.all(np.isfinite(res_p["out"]))
    np.testing.assert_array_equal(res_p["out"], res["out"])
    # weights sum to one: output of constant V is that constant (checked through lse sanity)
    assert np.all(np.isfinite(res["lse"]))


def test_bf16_encode_decode_roundtrip_and_rne():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.140625, 0.0], np.float32)
    u = workloads.encode(x, "bf16")
    back = consumers.decode(u, "bf16")
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even mantissa (1.0)
    assert back[1] == 1.0
    # 1.01171875 = 1 + 3*2^-8 is a tie between 1.0078125 and 1.015625 -> even (1.015625)
    assert back[2] == 1.015625
    assert back[0] == 1.0 and back[3] == -2.5 and back[4] == 3.140625 and back[5] == 0.0


# ------------------------------------------------------------------ producer-side store (Sec. 3.1, 4.2, 4.4)
def test_store_through_round_trip_and_untouched_elements():
    """Assigning to a virtual tensor and reading it back through the same chain returns the
    values; physical elements the map does not reach keep their contents (clone semantics of
    ScatterND's data input)."""
    rng = np.random.default_rng(0)
    src = {"A": rng.integers(0, 1000, size=(4, 6, 5)).astype(np.int64),
           "B": rng.integers(0, 1000, size=(3, 4)).astype(np.int64)}
    chain = [("a1", "slice", ("A",), {"dim": 1, "start": 1, "stop": 4}),          # [4,3,5]
             ("a2", "permute", ("a1",), {"perm": (1, 0, 2)}),                       # [3,4,5]
             ("a3", "reshape", ("a2",), {"shape": (3, 20)}),
             ("R", "concat", ("a3", "B"), {"dim": 1})]                             # [3,24]
    vals = np.arange(3 * 24).reshape(3, 24) + 5000
    out = dm_ops.store_through(chain, src, "R", vals)
    ch = index_maps.Chain(chain, {k: v.shape for k, v in src.items()})
    assert np.array_equal(ch.materialize_by_pull_back("R", out), vals)
    # written region of A is exactly the slice; the rest is the old data
    mask = np.zeros(src["A"].shape, bool)
    mask[:, 1:4, :] = True
    assert np.array_equal(out["A"][~mask], src["A"][~mask])
    assert (out["A"][mask] >= 5000).all() and (out["B"] >= 5000).all()
    # the same result from the operators written out one by one (Split, Transpose, slice assignment)
    a_part, b_part = vals[:, :20], vals[:, 20:]
    expect_a = src["A"].copy()
    expect_a[:, 1:4, :] = a_part.reshape(3, 4, 5).transpose(1, 0, 2)
    assert np.array_equal(out["A"], expect_a) and np.array_equal(out["B"], b_part)


def test_store_through_rejects_maps_that_are_not_one_to_one():
    src = {"A": np.zeros((2, 3), np.int64)}
    chain = [("u", "unsqueeze", ("A",), {"dim": 0}), ("e", "expand", ("u",), {"shape": (4, 2, 3)})]
    with pytest.raises(ValueError):
        dm_ops.store_through(chain, src, "e", np.zeros((4, 2, 3), np.int64))
    with pytest.raises(ValueError):
        dm_ops.store_through([("g", "index_select", ("A",), {"dim": 0, "index": "i"})], src, "g",
                             np.zeros((3, 3), np.int64), {"i": np.array([0, 1, 0], np.int32)})


@pytest.mark.parametrize("T", [1, 3])
def test_qkv_projection_store_equals_split_reshape_scatter(T):
    """Fig. 4 / Sec. 3.1: storing the merged projection through the virtual tensor equals
    Split into Q, K, V, Reshape, and ScatterND of K, V into the cache at positions pos .. pos+T-1."""
    B, Hq, Hkv, D, cap, pos, hidden = 2, 4, 2, 8, 16, 5, 32
    wl = workloads.qkv_proj_store(seed=3, B=B, hidden=hidden, Hq=Hq, Hkv=Hkv, D=D, cap=cap, pos=pos, T=T)
    res = run_workload(wl)
    c = consumers.round_to(res["out"], "bf16")                       # [B*T, (Hq+2Hkv)*D]
    q, k, v = c[:, :Hq * D], c[:, Hq * D:(Hq + Hkv) * D], c[:, (Hq + Hkv) * D:]
    assert np.array_equal(res["stored"]["Qbuf"], q.reshape(B, T, Hq * D))
    for name, part in (("Kcache", k), ("Vcache", v)):
        expect = wl.sources[name].copy()
        for b in range(B):
            for t in range(T):
                for h in range(Hkv):
                    expect[b, h, pos + t, :] = part[b * T + t, h * D:(h + 1) * D]    # ScatterND: one row per index
        assert np.array_equal(res["stored"][name], expect)
        assert not np.array_equal(expect, wl.sources[name])
    # and the product itself against a plain triple loop on a few entries
    a, w = consumers.decode(wl.sources["X"], "bf16"), consumers.decode(wl.sources["W"], "bf16")
    for (i, j) in [(0, 0), (B * T - 1, (Hq + 2 * Hkv) * D - 1), (1, Hq * D + 3)]:
        assert abs(sum(a[i, kk] * w[kk, j] for kk in range(hidden)) - res["out"][i, j]) < 1e-12


def test_round_to_bf16_is_round_to_nearest_even():
    # exact bf16 values stay; ties go to the even mantissa; the rest to the nearest
    def bits(f):
        return int(np.array([f], np.float32).view(np.uint32)[0] >> 16)
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0, 3.0e38])
    r = consumers.round_to(x, "bf16")
    assert list(r[:4]) == [bits(1.0), bits(1.0), bits(1.0 + 2.0 ** -6), bits(1.0 + 2.0 ** -7)]
    assert r[4] == bits(-2.5) and r[5] == 0
    assert np.array_equal(consumers.decode(r, "bf16")[:1], [1.0])
    # agrees with the input generator's rounding on random float32 values
    y = np.random.default_rng(1).standard_normal(4096).astype(np.float32)
    assert np.array_equal(consumers.round_to(y.astype(np.float64), "bf16"), workloads.encode(y, "bf16"))


# ------------------------------------------------------------------ mixture-of-experts combine
def test_moe_combine_routing_is_the_inverse_of_the_dispatch():
    """pos0/pos1 must name, in the expert-major buffer config 5 writes, exactly the two rows that
    hold token t: rebuilding that buffer's token ids from config 5's own tables pins them."""
    T, E = 500, 8
    wl = workloads.moe_combine(seed=7, T=T, E=E, N=16)
    d5 = workloads.c5_moe_dispatch(seed=7, T=T, Hd=8, E=E, N=8)
    token_of_row = np.concatenate([d5.index_tables["idx%d" % e] for e in range(E)])   # row of Y -> token
    assert token_of_row.shape == (2 * T,)
    p0, p1 = wl.index_tables["pos0"], wl.index_tables["pos1"]
    assert np.array_equal(token_of_row[p0], np.arange(T)) and np.array_equal(token_of_row[p1], np.arange(T))
    assert (p0 < p1).all()                                       # lower expert id first: distinct rows
    assert len(np.unique(np.concatenate([p0, p1]))) == 2 * T     # every row of Y is used exactly once
    w = wl.consumer["weights"]
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-6) and (w > 0).all()


def test_weighted_sum_against_a_plain_loop_and_special_weights():
    wl = workloads.moe_combine(seed=8, T=40, E=4, N=24)
    out = run_workload(wl)["out"]
    Y = consumers.decode(wl.sources["Y"], "bf16")
    w = wl.consumer["weights"].astype(np.float64)
    for t in (0, 17, 39):
        for c in (0, 23):
            want = w[t, 0] * Y[wl.index_tables["pos0"][t], c] + w[t, 1] * Y[wl.index_tables["pos1"][t], c]
            assert abs(out[t, c] - want) < 1e-12
    # weights (1, 0) return the first expert's row, (0, 1) the second's, (1, 1) on equal rows twice the row
    x = np.arange(12.0).reshape(3, 4)
    assert np.array_equal(consumers.weighted_sum(x, -x, np.array([[1, 0]] * 3, np.float32)), x)
    assert np.array_equal(consumers.weighted_sum(x, -x, np.array([[0, 1]] * 3, np.float32)), -x)
    assert np.array_equal(consumers.weighted_sum(x, x, np.array([[1, 1]] * 3, np.float32)), 2 * x)
