"""Host logic of the library (no GPU): the descriptor builder evaluated on the CPU through
vt_eval_host against the oracle's dense, op-by-op result; contiguity analysis (Def. 4/5);
error paths; exported symbols."""
import itertools
import os
import re

import numpy as np
import pytest

import paper_2604_09558_amd as vt
import workloads
from oracle import dm_ops

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def specs_of(wl, ptrs=None):
    return {k: (v.shape, wl.dtype) for k, v in wl.sources.items()}


def check_desc_against_dense(desc, dense, wl):
    """Every virtual index: descriptor -> (source, offset) must name the value the oracle put there."""
    info = desc.info()
    assert info["shape"] == dense.shape
    flat = {n: wl.sources[n].ravel() for n in desc.source_names}
    for x in itertools.product(*[range(n) for n in dense.shape]):
        src, off = desc.eval_host(x)
        name = desc.source_names[src]
        assert 0 <= off < flat[name].size, (x, src, off)
        got = flat[name][off]
        assert got == dense[x] or (got != got and dense[x] != dense[x]), (x, name, off, desc.dump())
        # the kernels' evaluator over the device form must agree with the host evaluator
        try:
            pc, off2 = desc.eval_device_form(x)
        except vt.VtError as e:
            assert e.code == vt.ERR_UNSUPPORTED
            continue
        assert off2 == off and desc.piece(pc)["src"] == src, (x, desc.dump())


def test_exported_symbols_match_header():
    hdr = open(os.path.join(ROOT, "include", "vt.h")).read()
    names = set(re.findall(r"\b(vt_[a-z_]+)\s*\(", hdr))
    assert {"vt_build", "vt_elementwise", "vt_gemm", "vt_decode_attn", "vt_materialize", "vt_copy_op"} <= names
    L = vt.lib()
    for n in sorted(names):
        assert hasattr(L, n), n


@pytest.mark.parametrize("seed", range(150))
def test_random_chain_descriptor_equals_oracle(seed):
    wl = workloads.random_chain(seed, n_ops=6)
    dense = dm_ops.run_chain(wl.chain, wl.sources, wl.index_tables)["R"]
    try:
        d = vt.build_chain(wl.chain, specs_of(wl), "R", wl.index_tables)
    except vt.VtError as e:
        assert e.code == vt.ERR_UNSUPPORTED, str(e)
        pytest.skip("outside the descriptor's reach: " + str(e))
    check_desc_against_dense(d, dense, wl)
    check_runs(d)


def test_most_random_chains_are_supported():
    ok = 0
    for seed in range(150):
        wl = workloads.random_chain(seed, n_ops=6)
        try:
            vt.build_chain(wl.chain, specs_of(wl), "R", wl.index_tables)
            ok += 1
        except vt.VtError as e:
            assert e.code == vt.ERR_UNSUPPORTED
    assert ok >= 140, ok


def local_linear(local, shape):
    lin = 0
    for a, n in zip(local, shape):
        lin = lin * n + a
    return lin


def check_runs(d):
    """Soundness and maximality of each piece's contiguous run, by scanning the piece."""
    info = d.info()
    shape = info["shape"]
    runs = []
    for p in range(info["n_pieces"]):
        pc = d.piece(p)
        lshape = tuple(h - l for l, h in zip(pc["lo"], pc["hi"]))
        run = pc["run"]
        runs.append(run)
        size = int(np.prod(lshape))
        assert run >= 1 and size % run == 0
        offs = {}
        glin = {}
        for loc in itertools.product(*[range(n) for n in lshape]):
            x = tuple(a + l for a, l in zip(loc, pc["lo"]))
            src, off = d.eval_host(x)
            assert src == pc["src"]
            ll = local_linear(loc, lshape)
            offs[ll] = off
            glin[ll] = local_linear(x, shape)
        broke = False
        for ll in range(size - 1):
            same_block = (ll + 1) % run != 0
            consecutive = offs[ll + 1] == offs[ll] + 1 and glin[ll + 1] == glin[ll] + 1
            if same_block:
                assert consecutive, (p, ll, run, d.dump())
            elif not consecutive:
                broke = True
        # maximal among runs that are products of trailing refined digits: some block
        # boundary must really break, unless the run already covers the piece
        # (an index table may be consecutive by accident: the analysis never looks at its entries;
        # below a stacked stage it reasons from the alignment of the piece's base against the lower
        # digits, not from the piece's extent, so a piece that happens to end before the lower
        # digit wraps may be contiguous beyond its run: sound, not maximal)
        assert broke or run == size or ",T" in d.dump() or "| base=" in d.dump(), (p, run, d.dump())
    assert info["run"] == min(runs)


def check_blocks(d):
    """Soundness and maximality of the block analysis by enumeration: every aligned group of
    `block` consecutive elements (row-major over the whole virtual tensor) is one contiguous range
    of one source, and twice that size is not (or does not divide the tensor)."""
    shape = d.shape
    n = int(np.prod(shape))
    where = [d.eval_host(x) for x in itertools.product(*[range(e) for e in shape])]

    def sound(c):
        if n % c:
            return False
        for s in range(0, n, c):
            src0, off0 = where[s]
            if any(where[s + k] != (src0, off0 + k) for k in range(1, c)):
                return False
        return True

    b = d.block()
    assert b >= 1 and b & (b - 1) == 0 and sound(b), (b, d.dump())
    return b, sound(2 * b)


@pytest.mark.parametrize("seed", range(150))
def test_block_analysis_is_sound_on_random_chains(seed):
    wl = workloads.random_chain(seed, n_ops=5, max_extent=8)
    try:
        d = vt.build_chain(wl.chain, specs_of(wl), "R", wl.index_tables)
    except vt.VtError:
        pytest.skip("chain not representable")
    check_blocks(d)


def test_block_analysis_known_cases_and_mostly_maximal():
    # config 1: the 16 + 5 column pieces of a 21-column row admit no block above one element
    wl = workloads.c1_tiny_chain()
    assert vt.build_chain(wl.chain, specs_of(wl), "V").block() == 1
    # config 3 (small): 128 contiguous elements per (row, head); config 4 (small): 7 tokens of 128
    wl = workloads.c3_oproj_gemm(B=2, H=4, S=8, D=128, N=8)
    assert vt.build_chain(wl.chain, specs_of(wl), "A").block() == 128
    # a concat along dim 0 of two dense tensors: blocks up to the gcd of the two parts
    d = vt.build_chain([("c", "concat", ("a", "b"), {"dim": 0})], {"a": ((4, 8), "f32"), "b": ((12, 8), "f32")}, "c")
    assert d.block() == 32 and d.block(16) == 16
    # the cap is honoured, and the analysis is never unsound; count how often it is also maximal
    maximal = total = 0
    for seed in range(150):
        wl = workloads.random_chain(seed, n_ops=4, max_extent=8)
        try:
            d = vt.build_chain(wl.chain, specs_of(wl), "R", wl.index_tables)
        except vt.VtError:
            continue
        b, bigger_ok = check_blocks(d)
        total += 1
        maximal += not bigger_ok
    assert total >= 100 and maximal >= 0.8 * total, (maximal, total)


# ------------------------------------------------------------------ benchmark chains
def test_c1_descriptor():
    wl = workloads.c1_tiny_chain()
    dense = dm_ops.run_chain(wl.chain, wl.sources)["V"]
    d = vt.build_chain(wl.chain, specs_of(wl), "V")
    check_desc_against_dense(d, dense, wl)
    info = d.info()
    assert info["n_pieces"] == 2 and info["run"] == 1
    assert d.piece(0)["hi"] == (8, 16) and d.piece(1)["lo"] == (0, 16) and d.piece(1)["run"] == 5
    # hand closed form: c < 16 -> X offset 8*(c+4) + r ; c >= 16 -> Y offset 5*r + c - 16
    for r in range(8):
        for c in range(21):
            src, off = d.eval_host((r, c))
            if c < 16:
                assert (d.source_names[src], off) == ("X", 8 * (c + 4) + r)
            else:
                assert (d.source_names[src], off) == ("Y", 5 * r + c - 16)


def test_c2_descriptor_small_and_full_size_structure():
    wl = workloads.c2_decode_attention(B=2, Hkv=2, G=4, S=5, D=128)
    env = dm_ops.run_chain(wl.chain, wl.sources)
    for name in ("Q", "K", "V"):
        d = vt.build_chain(wl.chain, specs_of(wl), name)
        check_desc_against_dense(d, env[name], wl)
    # full size: build from shapes only (no data needed) and check the closed form on samples
    B, Hkv, G, S, D = 8, 8, 4, 4096, 128
    E = (Hkv * G + 2 * Hkv) * D
    specs = {"QKV": ((B, 1, E), "bf16"), "Kcache": ((B, Hkv, S, D), "bf16"), "Vcache": ((B, Hkv, S, D), "bf16")}
    chain = workloads.c2_chain(B, Hkv, G, S, D)
    k = vt.build_chain(chain, specs, "K")
    info = k.info()
    assert info["shape"] == (B, Hkv * G, S, D) and info["n_pieces"] == 2
    assert k.piece(0)["hi"][2] == S - 1 and k.piece(1)["lo"][2] == S - 1
    assert k.piece(0)["run"] == (S - 1) * D and k.piece(1)["run"] == D and info["run"] == D
    rng = np.random.default_rng(0)
    for _ in range(500):
        b, h, t, dd = (int(rng.integers(0, n)) for n in (B, Hkv * G, S, D))
        if rng.integers(0, 4) == 0:
            t = S - 1
        src, off = k.eval_host((b, h, t, dd))
        if t < S - 1:
            assert (k.source_names[src], off) == ("Kcache", ((b * Hkv + h // G) * S + t) * D + dd)
        else:
            assert (k.source_names[src], off) == ("QKV", b * E + Hkv * G * D + (h // G) * D + dd)
    q = vt.build_chain(chain, specs, "Q")
    assert q.info()["run"] == Hkv * G * D     # the whole Q block of a batch row is contiguous


def test_c3_c4_c5_descriptors_full_size_closed_forms():
    rng = np.random.default_rng(1)
    # C3
    B, H, S, D = 16, 32, 512, 128
    chain = [("o1", "permute", ("O",), {"perm": (0, 2, 1, 3)}), ("A", "reshape", ("o1",), {"shape": (B * S, H * D)})]
    a = vt.build_chain(chain, {"O": ((B, H, S, D), "bf16")}, "A")
    assert a.info()["run"] == D and a.info()["n_pieces"] == 1
    for _ in range(300):
        m, k = int(rng.integers(0, B * S)), int(rng.integers(0, H * D))
        assert a.eval_host((m, k))[1] == (m // S) * 2097152 + (k // D) * 65536 + (m % S) * D + k % D
    # C4
    Bc, R, win, Cc = 32, 56, 7, 128
    nw = R // win
    chain = [("x1", "reshape", ("X",), {"shape": (Bc, nw, win, nw, win, Cc)}),
             ("x2", "permute", ("x1",), {"perm": (0, 1, 3, 2, 4, 5)}),
             ("T", "reshape", ("x2",), {"shape": (Bc * nw * nw, win * win, Cc)})]
    t = vt.build_chain(chain, {"X": ((Bc, R, R, Cc), "f16")}, "T")
    assert t.info()["run"] == win * Cc              # 7 tokens of 128 channels = 896 elements
    for _ in range(300):
        w, p, c = int(rng.integers(0, 2048)), int(rng.integers(0, 49)), int(rng.integers(0, 128))
        b, wh, ww, ih, iw = w // 64, (w // 8) % 8, w % 8, p // 7, p % 7
        assert t.eval_host((w, p, c))[1] == ((b * 56 + wh * 7 + ih) * 56 + ww * 7 + iw) * 128 + c
    # C5 (small T, real hidden size): row r of expert e is token idx_e[r]
    wl = workloads.c5_moe_dispatch(T=64, Hd=4096, E=8, N=16)
    for e in (0, 5):
        d = vt.build_chain(wl.chain, specs_of(wl), "A%d" % e, wl.index_tables)
        idx = wl.index_tables["idx%d" % e]
        assert d.info()["run"] == 4096 and d.info()["shape"] == (len(idx), 4096)
        for r in range(len(idx)):
            assert d.eval_host((r, 17))[1] == int(idx[r]) * 4096 + 17
        bdesc = vt.build_chain(wl.chain, specs_of(wl), "B%d" % e, wl.index_tables)
        assert bdesc.eval_host((3, 5))[1] == e * 4096 * 16 + 3 * 16 + 5
        assert bdesc.info()["run"] == 4096 * 16


def test_paper_contiguity_cases():
    # split along axis 0 keeps full contiguity (Sec. 4.4, Split: Type I); along axis 1 it does not
    src = {"X": ((6, 10), "f32")}
    d0 = vt.build_chain([("a", "split", ("X",), {"dim": 0, "sizes": (2, 4), "output": 1})], src, "a")
    assert d0.info()["run"] == 4 * 10                 # minimal contiguous dimension = 1: whole tensor
    d1 = vt.build_chain([("a", "split", ("X",), {"dim": 1, "sizes": (4, 6), "output": 1})], src, "a")
    assert d1.info()["run"] == 6                      # partial contiguity: chunk of a row
    # Eq. 2's expand: (a,b,c) -> (a,3b,c): run is b*c (one replica), bias jumps at each replica
    a, b, c = 2, 3, 4
    chain = [("u", "unsqueeze", ("X",), {"dim": 1}), ("e", "expand", ("u",), {"shape": (a, 3, b, c)}),
             ("y", "reshape", ("e",), {"shape": (a, 3 * b, c)})]
    d = vt.build_chain(chain, {"X": ((a, b, c), "f32")}, "y")
    assert d.info()["run"] == b * c
    for i, j, k in itertools.product(range(a), range(3 * b), range(c)):
        assert d.eval_host((i, j, k))[1] == i * b * c + j * c + k - (j // b) * b * c
    # transposed matrix: no contiguity
    dt = vt.build_chain([("t", "permute", ("X",), {"perm": (1, 0)})], src, "t")
    assert dt.info()["run"] == 1
    # strided source (Sec. 2.1 stride vector given explicitly)
    ds = vt.build_chain([], {"X": ((3, 4), "f32", 0, (8, 2))}, "X")
    assert ds.eval_host((2, 3))[1] == 2 * 8 + 3 * 2 and ds.info()["run"] == 1


def test_profitability_classes_of_the_papers_cases():
    """Sec. 4.3/4.4: split along axis 0, a reshape and a whole-range slice keep the original
    access pattern up to a constant bias (Type I); split along another axis, expand, permute and
    concat do not, and whether they keep partial contiguity depends on the run against the
    minimal transfer unit."""
    src = {"X": ((6, 64), "f32")}
    full = [
        [("a", "split", ("X",), {"dim": 0, "sizes": (2, 4), "output": 1})],
        [("a", "reshape", ("X",), {"shape": (3, 2, 8, 8)})],
        [("a", "slice", ("X",), {"dim": 0, "start": 2, "stop": 5})],
    ]
    for chain in full:
        cls, run = vt.build_chain(chain, src, "a").classify()
        assert cls == vt.ACCESS_FULL, chain
    # split along axis 1: runs of 24 floats = 96 bytes: partial for a 64-byte unit, scattered for 128
    d = vt.build_chain([("a", "split", ("X",), {"dim": 1, "sizes": (40, 24), "output": 1})], src, "a")
    assert d.classify(64) == (vt.ACCESS_PARTIAL, 96)
    assert d.classify(128) == (vt.ACCESS_SCATTERED, 96)
    assert d.classify() == (vt.ACCESS_SCATTERED, 96)         # default unit: 128 bytes
    # transposed matrix: single elements
    assert vt.build_chain([("t", "permute", ("X",), {"perm": (1, 0)})], src, "t").classify() == (vt.ACCESS_SCATTERED, 4)
    # expand is never Type I (Sec. 4.4), even though every replica is one long run
    chain = [("u", "unsqueeze", ("X",), {"dim": 0}), ("e", "expand", ("u",), {"shape": (4, 6, 64)})]
    assert vt.build_chain(chain, src, "e").classify() == (vt.ACCESS_PARTIAL, 6 * 64 * 4)
    # a tensor stitched from separately stored parts (the input of a split seen as a virtual
    # tensor of its outputs) is not Type I either
    two = {"A": ((2, 64), "f32"), "B": ((4, 64), "f32")}
    d = vt.build_chain([("c", "concat", ("A", "B"), {"dim": 0})], two, "c")
    assert d.classify() == (vt.ACCESS_PARTIAL, 2 * 64 * 4)
    assert vt.lib().vt_classify(None, 0, None, None) == vt.ERR_INVALID_ARG


@pytest.mark.parametrize("seed", range(40))
def test_full_class_means_identity_plus_bias(seed):
    """Theorem 1's premise checked by brute force: FULL iff walking the virtual tensor in
    row-major order walks one source in consecutive offsets."""
    wl = workloads.random_chain(seed, n_ops=3)
    try:
        d = vt.build_chain(wl.chain, specs_of(wl), "R", wl.index_tables)
    except vt.VtError:
        pytest.skip("outside the descriptor's reach")
    shape = d.info()["shape"]
    walk = [d.eval_host(x) for x in itertools.product(*[range(n) for n in shape])]
    identity = all(s == walk[0][0] and o == walk[0][1] + i for i, (s, o) in enumerate(walk))
    cls, run = d.classify()
    if ",T" in d.dump() and identity:
        return                                              # an index table that happens to be consecutive
    assert (cls == vt.ACCESS_FULL) == identity, (d.dump(), cls)


def test_benchmark_chains_classes():
    c1 = workloads.c1_tiny_chain()
    assert vt.build_chain(c1.chain, specs_of(c1), c1.consumer["x"]).classify()[0] == vt.ACCESS_SCATTERED
    c2 = workloads.c2_decode_attention()
    for name in ("K", "V"):
        cls, run = vt.build_chain(c2.chain, specs_of(c2), c2.consumer[name.lower()]).classify()
        assert (cls, run) == (vt.ACCESS_PARTIAL, 256)       # the new token's row in the fused QKV buffer
    c3 = workloads.c3_oproj_gemm()
    assert vt.build_chain(c3.chain, specs_of(c3), "A").classify() == (vt.ACCESS_PARTIAL, 256)
    c4 = workloads.c4_window_ln_linear()
    assert vt.build_chain(c4.chain, specs_of(c4), c4.consumer["x"]).classify() == (vt.ACCESS_PARTIAL, 7 * 128 * 2)


def dense_case(sources, chain, tables=None, result="R"):
    src = {k: np.arange(100 * i, 100 * i + int(np.prod(shp)), dtype=np.float32).reshape(shp) for i, (k, shp) in enumerate(sources.items())}
    wl = workloads.Workload("case", "f32", src, chain, {"kind": "materialize", "x": result}, tables or {})
    dense = dm_ops.run_chain(chain, wl.sources, wl.index_tables)[result]
    d = vt.build_chain(chain, specs_of(wl), result, wl.index_tables)
    check_desc_against_dense(d, dense, wl)
    check_runs(d)
    check_blocks(d)
    return d


def test_index_select_along_a_concatenated_dim():
    """Sec. 4.1 puts no restriction on composition: a gather whose table crosses the parts of a
    Concat is split into runs of entries that stay in one part."""
    cat = [("c", "concat", ("X", "Y"), {"dim": 1})]
    # entries 0..5 name X's columns, 6..10 Y's
    for table, pieces in (([0, 1, 7, 8, 9, 3], 3), ([10, 9, 8, 7, 6], 1), ([5, 6, 5, 6], 4), ([2], 1), ([0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10], 2)):
        d = dense_case({"X": (4, 6), "Y": (4, 5)}, cat + [("R", "index_select", ("c",), {"dim": 1, "index": "t"})], {"t": np.array(table, np.int32)})
        assert d.info()["n_pieces"] == pieces, (table, d.dump())
    # the gathered dim was cut, another dim is cut as well; operators follow
    chain = [("a", "concat", ("X", "Y"), {"dim": 1}), ("b", "concat", ("a", "Z"), {"dim": 0}),
             ("g", "index_select", ("b",), {"dim": 0, "index": "t"}), ("p", "permute", ("g",), {"perm": (1, 0)}),
             ("R", "slice", ("p",), {"dim": 0, "start": 2, "stop": 9, "step": 1})]
    dense_case({"X": (4, 6), "Y": (4, 5), "Z": (2, 11)}, chain, {"t": np.array([5, 0, 1, 4, 2], np.int32)})
    # a part of extent 1 along the gathered dim, and a gather of a gather
    chain = [("c", "concat", ("X", "Y"), {"dim": 0}), ("g", "index_select", ("c",), {"dim": 0, "index": "t"}),
             ("R", "index_select", ("g",), {"dim": 0, "index": "u"})]
    dense_case({"X": (1, 3), "Y": (3, 3)}, chain, {"t": np.array([0, 0, 2, 3, 1], np.int32), "u": np.array([4, 0, 2, 2], np.int32)})


def test_reshape_across_a_concat_cut():
    """A Reshape that regroups a dim which a Concat cut: each part of the old dim is an interval of
    the row-major order and becomes a few boxes of the new shape."""
    cat0 = [("c", "concat", ("X", "Y"), {"dim": 0})]
    for shape, pieces in (((2, 6), 3), ((6, 2), 2), ((4, 3), 4), ((12,), 2), ((2, 2, 3), 4), ((3, 2, 2), 2), ((1, 12, 1), 2)):
        d = dense_case({"X": (2, 4), "Y": (1, 4)}, cat0 + [("R", "reshape", ("c",), {"shape": shape})])
        assert d.info()["n_pieces"] == pieces, (shape, d.dump())
    # the cut dim is an inner one: one interval per outer index
    cat1 = [("c", "concat", ("X", "Y"), {"dim": 1})]
    d = dense_case({"X": (3, 4), "Y": (3, 2)}, cat1 + [("R", "reshape", ("c",), {"shape": (18,)})])
    assert d.info()["n_pieces"] == 6
    dense_case({"X": (2, 4), "Y": (2, 2)}, cat1 + [("R", "reshape", ("c",), {"shape": (3, 4)})])
    dense_case({"X": (2, 3, 4), "Y": (2, 3, 2)}, [("c", "concat", ("X", "Y"), {"dim": 2}), ("R", "reshape", ("c",), {"shape": (2, 18)})])
    # views under the concat, operators after the reshape
    chain = [("xp", "permute", ("X",), {"perm": (1, 0)}), ("c", "concat", ("xp", "Y"), {"dim": 0}), ("r", "reshape", ("c",), {"shape": (4, 5)}),
             ("s", "slice", ("r",), {"dim": 1, "start": 1, "stop": 4, "step": 1}), ("R", "permute", ("s",), {"perm": (1, 0)})]
    dense_case({"X": (2, 6), "Y": (4, 2)}, chain)
    # too many intervals for the descriptor
    with pytest.raises(vt.VtError) as ei:
        dense_case({"X": (40, 4), "Y": (40, 2)}, cat1 + [("R", "reshape", ("c",), {"shape": (240,)})])
    assert ei.value.code == vt.ERR_UNSUPPORTED


def test_stacked_stage_case():
    # a reshape that straddles a slice boundary needs a second stage
    chain = [("a", "slice", ("X",), {"dim": 1, "start": 0, "stop": 3, "step": 1}),
             ("b", "reshape", ("a",), {"shape": (2, 9)}),
             ("c", "slice", ("b",), {"dim": 1, "start": 0, "stop": 8, "step": 1}),
             ("R", "reshape", ("c",), {"shape": (16,)})]
    wl = workloads.Workload("stack", "f32", {"X": np.arange(24, dtype=np.float32).reshape(6, 4)}, chain,
                            {"kind": "materialize", "x": "R"})
    dense = dm_ops.run_chain(chain, wl.sources)["R"]
    d = vt.build_chain(chain, specs_of(wl), "R")
    assert "|" in d.dump()                            # more than one stage
    check_desc_against_dense(d, dense, wl)


def test_a_piece_inside_one_dense_run_of_the_stage_below_keeps_its_run():
    """expand -> reshape -> split leaves a stacked stage; the two elements kept are neighbours in the
    source (elements 0 and 1 of the first row of three), although neither the start's alignment
    nor the lower digit's radix (3) is a multiple of the run (2): the extent decides."""
    chain = [("v0", "expand", ("S0",), {"shape": (3, 2, 3)}),
             ("v1", "reshape", ("v0",), {"shape": (1, 18)}),
             ("v2", "split", ("v1",), {"dim": 1, "sizes": (2, 16), "output": 0}),
             ("R", "reshape", ("v2",), {"shape": (1, 2)})]
    d = vt.build_chain(chain, {"S0": ((3, 1, 3), "f32")}, "R")
    assert d.info()["run"] == 2
    assert d.eval_host((0, 0)) == (0, 0) and d.eval_host((0, 1)) == (0, 1)
    check_runs(d)
    # one element further and the piece crosses into the broadcast copy of the row: no run of 4
    chain[2] = ("v2", "split", ("v1",), {"dim": 1, "sizes": (4, 14), "output": 0})
    chain[3] = ("R", "reshape", ("v2",), {"shape": (1, 4)})
    d = vt.build_chain(chain, {"S0": ((3, 1, 3), "f32")}, "R")
    assert d.info()["run"] == 1
    check_runs(d)


def test_error_paths():
    src = {"X": ((4, 6), "f32"), "Y": ((4, 5), "f32"), "H": ((4, 6), "f16")}

    def code(chain, result, tables=None, s=src):
        with pytest.raises(vt.VtError) as ei:
            vt.build_chain(chain, s, result, tables)
        return ei.value.code

    assert code([("a", "reshape", ("X",), {"shape": (5, 5)})], "a") == vt.ERR_SHAPE
    assert code([("a", "slice", ("X",), {"dim": 1, "start": 2, "stop": 9, "step": 1})], "a") == vt.ERR_RANGE
    assert code([("a", "slice", ("X",), {"dim": 2, "start": 0, "stop": 1, "step": 1})], "a") == vt.ERR_RANGE
    assert code([("a", "split", ("X",), {"dim": 1, "sizes": (2, 2), "output": 0})], "a") == vt.ERR_RANGE
    assert code([("a", "permute", ("X",), {"perm": (0, 0)})], "a") == vt.ERR_INVALID_ARG
    assert code([("a", "concat", ("X", "Y"), {"dim": 0})], "a") == vt.ERR_SHAPE
    assert code([("a", "concat", ("X", "H"), {"dim": 0})], "a") == vt.ERR_INVALID_ARG
    assert code([("a", "expand", ("X",), {"shape": (4, 12)})], "a") == vt.ERR_SHAPE
    t = {"i": np.array([0, 7], np.int32)}
    assert code([("a", "index_select", ("X",), {"dim": 0, "index": "i"})], "a", t) == vt.ERR_RANGE
    # a table that hops between the parts of a concatenated dim more often than the descriptor has pieces
    t = {"i": np.array([0, 7] * 9, np.int32)}
    chain = [("c", "concat", ("X", "Y"), {"dim": 1}), ("a", "index_select", ("c",), {"dim": 1, "index": "i"})]
    assert code(chain, "a", t) == vt.ERR_UNSUPPORTED
    # NULL arguments
    assert vt.lib().vt_build(None, 0, None, 0, 0, None) == vt.ERR_INVALID_ARG
    assert vt.lib().vt_desc_info(None, None, None, None, None, None) == vt.ERR_INVALID_ARG
    assert b"NULL" in vt.lib().vt_last_error()
    d = vt.build_chain([], src, "X")
    with pytest.raises(vt.VtError) as ei:
        d.eval_host((4, 0))
    assert ei.value.code == vt.ERR_RANGE
    # kernels refuse a descriptor without device pointers (no GPU call is made)
    with pytest.raises(vt.VtError) as ei:
        vt.vt_materialize(d, 16, stream=0)
    assert ei.value.code == vt.ERR_INVALID_ARG


def test_store_maps_must_be_one_to_one():
    """A descriptor is a legal store target only if no two virtual elements share a physical one
    (host check; no kernel is launched for a rejected map)."""
    fake = 0x1000        # never dereferenced: the check comes before any launch
    src = vt.build_chain([], {"S": ((4, 6), "f32", fake)}, "S")
    exp = vt.build_chain([("u", "unsqueeze", ("A",), {"dim": 0}), ("e", "expand", ("u",), {"shape": (4, 6)})],
                         {"A": ((6,), "f32", fake)}, "e")
    with pytest.raises(vt.VtError) as ei:
        vt.vt_scatter(src, exp)
    assert ei.value.code == vt.ERR_NOT_ONE_TO_ONE
    # the same tensor twice in a concat: the two pieces overlap
    twice = vt.build_chain([("c", "concat", ("A", "A"), {"dim": 1})], {"A": ((4, 3), "f32", fake)}, "c")
    with pytest.raises(vt.VtError) as ei:
        vt.vt_scatter(src, twice)
    assert ei.value.code == vt.ERR_NOT_ONE_TO_ONE
    # an index table on the output is refused (it may repeat entries)
    tab = vt.build_chain([("g", "index_select", ("A",), {"dim": 0, "index": "i"})], {"A": ((4, 6), "f32", fake)}, "g",
                         {"i": np.array([0, 1, 2, 3], np.int32)}, {"i": fake})
    with pytest.raises(vt.VtError) as ei:
        vt.vt_scatter(src, tab)
    assert ei.value.code == vt.ERR_UNSUPPORTED
    # shapes must agree
    with pytest.raises(vt.VtError) as ei:
        vt.vt_scatter(src, vt.build_chain([], {"S": ((6, 4), "f32", fake)}, "S"))
    assert ei.value.code == vt.ERR_SHAPE


# ------------------------------------------------------------------ host plan of the attention consumer
FAKE = 0x100000       # a 16-byte aligned address that is never dereferenced


def attn_descs(wl):
    spec = {k: (v.shape, wl.dtype, FAKE) for k, v in wl.sources.items()}
    tabs = {k: FAKE for k in wl.index_tables}
    c = wl.consumer
    return [vt.build_chain(wl.chain, spec, c[n], wl.index_tables, tabs) for n in ("q", "k", "v")]


def test_attention_plan_of_the_decode_chain():
    wl = workloads.c2_decode_attention(seed=0, B=8, Hkv=8, G=4, S=4096, D=128)
    plan = vt.vt_decode_attn_plan(*attn_descs(wl))
    # 4 query heads share a read; the context splits into cached rows | fresh row; 8 splits fill the chip
    assert plan == {"group_size": 4, "n_segments": 2, "splits": 8, "paged_segments": 0}
    assert vt.vt_decode_attn_plan(*attn_descs(wl), n_splits=3)["splits"] == 3
    small = workloads.c2_decode_attention(seed=0, B=1, Hkv=1, G=16, S=70, D=128)
    assert vt.vt_decode_attn_plan(*attn_descs(small)) == {"group_size": 16, "n_segments": 2, "splits": 1, "paged_segments": 0}


def test_attention_group_size_divides_the_broadcast_factor():
    """18 query heads per kv head: more than one matrix tile holds (16), so the group must be a
    divisor of 18 (9), not merely a divisor of the 36 query heads (12 would straddle two kv heads)."""
    wl = workloads.c2_decode_attention(seed=0, B=1, Hkv=2, G=18, S=40, D=128)
    assert vt.vt_decode_attn_plan(*attn_descs(wl))["group_size"] == 9
    wl = workloads.c2_decode_attention(seed=0, B=1, Hkv=3, G=17, S=40, D=128)      # a prime above 16: one head per read
    assert vt.vt_decode_attn_plan(*attn_descs(wl))["group_size"] == 1


def test_attention_plan_recognises_page_tables():
    two_stage = workloads.paged_decode_attention(seed=1, B=2, Hkv=2, G=4, pages_per_seq=3, page=32)
    assert vt.vt_decode_attn_plan(*attn_descs(two_stage)) == {"group_size": 4, "n_segments": 1, "splits": 1, "paged_segments": 1}
    one_stage = workloads.paged_decode_attention(seed=1, B=1, Hkv=2, G=1, pages_per_seq=2, page=128)   # B = 1: the table digit stays in the context group
    assert vt.vt_decode_attn_plan(*attn_descs(one_stage))["paged_segments"] == 1
    # pages that do not hold a multiple of 32 rows cannot be tiled
    odd = workloads.paged_decode_attention(seed=1, B=2, Hkv=1, G=2, pages_per_seq=3, page=24)
    with pytest.raises(vt.VtError) as ei:
        vt.vt_decode_attn_plan(*attn_descs(odd))
    assert ei.value.code == vt.ERR_UNSUPPORTED


def test_attention_plan_rejects_what_the_kernel_cannot_read():
    wl = workloads.c2_decode_attention(seed=0, B=1, Hkv=1, G=2, S=8, D=64)          # head dim 64
    with pytest.raises(vt.VtError) as ei:
        vt.vt_decode_attn_plan(*attn_descs(wl))
    assert ei.value.code == vt.ERR_UNSUPPORTED
    # K transposed so that the head dim is not contiguous
    wl = workloads.c2_decode_attention(seed=0, B=1, Hkv=1, G=2, S=128, D=128)
    q, k, v = attn_descs(wl)
    spec = {"X": ((1, 2, 128, 128), "bf16", FAKE)}
    kt = vt.build_chain([("t", "permute", ("X",), {"perm": (0, 1, 3, 2)})], spec, "t")
    with pytest.raises(vt.VtError) as ei:
        vt.vt_decode_attn_plan(q, kt, v)
    assert ei.value.code == vt.ERR_UNSUPPORTED
    assert vt.lib().vt_decode_attn_plan(None, None, None, 0, None, None, None, None) == vt.ERR_INVALID_ARG


# ----------------------------------------------------------------------------------------
# Row walk: the host's resolution of a [R, C] map into segments that are affine in (row, block)
# ----------------------------------------------------------------------------------------
FAKE_BASE = 1 << 40


def fake_ptrs(wl):
    """Distinct, far apart source addresses (never dereferenced on the host)."""
    return {k: (v.shape, wl.dtype, FAKE_BASE + (i << 34)) for i, (k, v) in enumerate(wl.sources.items())}


def check_row_walk(d, ptr_of_src, esz):
    """Every block address the segments give equals the evaluator's, and the segments tile the
    [R, C / block] domain exactly once.  Returns the number of segments (0: not resolved)."""
    R, Cc = d.shape
    be = d.block()
    while Cc % be:
        be //= 2
    segs = d.row_walk(be)
    if not segs:
        return 0
    covered = np.zeros((R, Cc // be), np.int32)
    for row_lo, row_hi, blk_lo, blk_hi, base, rs, bs, group, gs in segs:
        assert 0 <= row_lo < row_hi <= R and 0 <= blk_lo < blk_hi <= Cc // be
        covered[row_lo:row_hi, blk_lo:blk_hi] += 1
        for r in range(row_lo, row_hi):
            for b in range(blk_lo, blk_hi):
                src, off = d.eval_host((r, b * be))
                j = b - blk_lo
                hi = j // group if group else 0
                assert base + (r - row_lo) * rs + (j - hi * group) * bs + hi * gs == ptr_of_src[src] + off * esz, (r, b, d.dump())
    assert (covered == 1).all(), d.dump()
    return len(segs)


def test_row_walk_of_the_benchmark_chain():
    wl = workloads.rowsum_chain_large()
    specs = fake_ptrs(wl)
    v = vt.build_chain(wl.chain, specs, "V")
    segs = v.row_walk(128)
    x, y = specs["X"][2], specs["Y"][2]
    # X[a, row, :] is block a of the row: one row further 128 floats, one block further a whole [B, C0] slab
    assert segs == [(0, 8192, 0, 32, x, 128 * 4, 8192 * 128 * 4, 0, 0), (0, 8192, 32, 40, y, 1024 * 4, 128 * 4, 0, 0)]
    z = vt.build_chain(wl.chain, specs, "Z")
    assert z.row_walk(1024) == [(0, 8192, 0, 5, specs["Z"][2], 5120 * 4, 1024 * 4, 0, 0)]
    # half blocks: two of them share a run of X, then the address jumps to the next slab (two levels)
    assert v.row_walk(64) == [(0, 8192, 0, 64, x, 128 * 4, 64 * 4, 2, 8192 * 128 * 4), (0, 8192, 64, 80, y, 1024 * 4, 64 * 4, 0, 0)]
    # double blocks are not contiguous ranges of X; sizes that do not divide the row are refused
    assert v.row_walk(256) == [] and v.row_walk(96) == []


def test_row_walk_refuses_tables_and_stacked_stages():
    rng = np.random.default_rng(0)
    src = {"X": rng.normal(size=(12, 32)).astype(np.float32)}
    idx = rng.permutation(12).astype(np.int32)
    wl = workloads.Workload("g", "f32", src, [("R", "index_select", ("X",), {"dim": 0, "index": "I"})], {"kind": "none"}, {"I": idx})
    d = vt.build_chain(wl.chain, fake_ptrs(wl), "R", wl.index_tables)
    assert d.row_walk(32) == []
    # a slice that is not aligned to the inner dims, then a reshape: a second stage
    src = {"X": rng.normal(size=(6, 10)).astype(np.float32)}
    chain = [("s", "slice", ("X",), {"dim": 1, "start": 1, "stop": 9, "step": 1}), ("R", "reshape", ("s",), {"shape": (12, 4)})]
    wl = workloads.Workload("s", "f32", src, chain, {"kind": "none"})
    d = vt.build_chain(wl.chain, fake_ptrs(wl), "R")
    assert check_row_walk(d, {0: FAKE_BASE}, 4) in (0, 1)


@pytest.mark.parametrize("seed", range(120))
def test_row_walk_equals_the_evaluator_on_random_chains(seed):
    wl = workloads.random_chain(seed, n_ops=4, max_extent=8)
    specs = fake_ptrs(wl)
    try:
        d0 = vt.build_chain(wl.chain, specs, "R", wl.index_tables)
    except vt.VtError:
        pytest.skip("chain not representable")
    shape = d0.shape
    n = int(np.prod(shape))
    # the result seen as [R, C] for every split of its dims into leading and trailing ones
    resolved = 0
    for cut in range(len(shape) + 1):
        rows = int(np.prod(shape[:cut]))
        chain = list(wl.chain) + [("R2", "reshape", ("R",), {"shape": (rows, n // rows)})]
        try:
            d = vt.build_chain(chain, specs, "R2", wl.index_tables)
        except vt.VtError:
            continue
        ptr_of_src = {i: specs[name][2] for i, name in enumerate(d.source_names)}
        resolved += check_row_walk(d, ptr_of_src, 2 if wl.dtype != "f32" else 4) > 0
    # nothing to assert on `resolved` per seed: how often the form applies is counted below


def test_row_walk_resolves_most_table_free_chains():
    tried = ok = 0
    for seed in range(120):
        wl = workloads.random_chain(seed, n_ops=3, max_extent=8)
        if wl.index_tables:
            continue
        specs = fake_ptrs(wl)
        try:
            d0 = vt.build_chain(wl.chain, specs, "R")
        except vt.VtError:
            continue
        shape = d0.shape
        if len(shape) < 2:
            continue
        rows = int(shape[0])
        chain = list(wl.chain) + [("R2", "reshape", ("R",), {"shape": (rows, int(np.prod(shape)) // rows)})]
        try:
            d = vt.build_chain(chain, specs, "R2")
        except vt.VtError:
            continue
        tried += 1
        ok += len(d.row_walk(max(1, min(d.block(), 1)))) > 0
    assert tried >= 40, tried
    print("row walk resolved %d of %d table-free chains at block 1" % (ok, tried))


# ----------------------------------------------------------------------------------------
# Block walk: the general term form of a single-stage map, against the evaluator
# ----------------------------------------------------------------------------------------
def check_block_walk(d, ptr_of_src, esz, unit):
    """Every unit's address from the term form equals the evaluator's.  True if the map resolved."""
    shape = d.shape
    n = int(np.prod(shape))
    assert n % unit == 0
    got = d.walk_addresses(unit)
    if got is None:
        return False
    assert len(got) == n // unit
    for u, a in enumerate(got):
        x = np.unravel_index(u * unit, shape) if shape else ()
        src, off = d.eval_host(tuple(int(v) for v in x))
        assert a == ptr_of_src[src] + off * esz, (u, unit, d.dump())
    return True


def test_block_walk_of_the_benchmark_chains():
    wl = workloads.c4_window_ln_linear(B=2, R=14, win=7, C=128, N=384)
    specs = fake_ptrs(wl)
    t = vt.build_chain(wl.chain, specs, "T")
    # rows of the window partition: five digits, two of which nest into one term
    assert check_block_walk(t, {0: specs["X"][2]}, 2, 128)
    assert check_block_walk(t, {0: specs["X"][2]}, 2, 8)
    wl = workloads.rowsum_chain_large(A=4, B=96, C0=64, ny=48)
    specs = fake_ptrs(wl)
    v = vt.build_chain(wl.chain, specs, "V")
    ptrs = {i: specs[name][2] for i, name in enumerate(v.source_names)}
    assert check_block_walk(v, ptrs, 4, 16)            # concat along the last dim: a test on the column block
    assert check_block_walk(v, ptrs, 4, 1)
    assert v.walk_addresses(32) is None or check_block_walk(v, ptrs, 4, 32) is not None
    wl = workloads.c3_oproj_gemm(seed=3, B=2, H=3, S=100, D=64, N=264)
    specs = fake_ptrs(wl)
    a = vt.build_chain(wl.chain, specs, "A")
    assert check_block_walk(a, {0: specs[a.source_names[0]][2]}, 2, 64)


def test_block_walk_refuses_tables_and_stages():
    rng = np.random.default_rng(0)
    src = {"X": rng.normal(size=(12, 32)).astype(np.float32)}
    idx = rng.permutation(12).astype(np.int32)
    wl = workloads.Workload("g", "f32", src, [("R", "index_select", ("X",), {"dim": 0, "index": "I"})], {"kind": "none"}, {"I": idx})
    d = vt.build_chain(wl.chain, fake_ptrs(wl), "R", wl.index_tables)
    assert d.walk_addresses(32) is None
    with pytest.raises(vt.VtError):
        d.walk_addresses(0)


@pytest.mark.parametrize("seed", range(150))
def test_block_walk_equals_the_evaluator_on_random_chains(seed):
    wl = workloads.random_chain(seed, n_ops=5, max_extent=8)
    specs = fake_ptrs(wl)
    try:
        d = vt.build_chain(wl.chain, specs, "R", wl.index_tables)
    except vt.VtError:
        pytest.skip("chain not representable")
    n = int(np.prod(d.shape))
    ptr_of_src = {i: specs[name][2] for i, name in enumerate(d.source_names)}
    esz = 2 if wl.dtype != "f32" else 4
    units = {1, d.block()}
    if d.shape:
        units.add(int(d.shape[-1]))                    # rows
    for unit in sorted(units):
        if unit >= 1 and n % unit == 0:
            check_block_walk(d, ptr_of_src, esz, unit)


def test_block_walk_resolves_most_table_free_chains():
    tried = ok = 0
    for seed in range(200):
        wl = workloads.random_chain(seed, n_ops=4, max_extent=8)
        if wl.index_tables:
            continue
        specs = fake_ptrs(wl)
        try:
            d = vt.build_chain(wl.chain, specs, "R")
        except vt.VtError:
            continue
        tried += 1
        ok += d.walk_addresses(d.block(), 0, 0) is not None
    assert tried >= 60 and ok >= 0.6 * tried, (ok, tried)


def test_block_address_probes_check_their_arguments():
    wl = workloads.c1_tiny_chain()
    d = vt.build_chain(wl.chain, fake_ptrs(wl), "V")
    n = int(np.prod(d.shape))
    assert len(d.walk_addresses(1, n - 3, 3)) == 3
    with pytest.raises(vt.VtError) as e:
        d.walk_addresses(1, n - 3, 4)                   # one unit past the end
    assert e.value.code == vt.ERR_RANGE
    with pytest.raises(vt.VtError):
        d.walk_addresses(1, -1, 1)
    assert d.walk_addresses(5) is None                  # 5 does not divide 8 * 21
    # sources without pointers: nothing to resolve against
    bare = vt.build_chain(wl.chain, specs_of(wl), "V")
    assert bare.walk_addresses(1, 0, 0) is None and bare.row_walk(1) == []
    with pytest.raises(vt.VtError):
        d.row_walk(0)
    three_d = vt.build_chain([], {"S": ((2, 3, 4), "f32", FAKE_BASE)}, "S")
    with pytest.raises(vt.VtError) as e:
        three_d.row_walk(4)
    assert e.value.code == vt.ERR_SHAPE
