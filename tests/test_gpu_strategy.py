"""Workloads run under arbitrary virtual tensor strategies (Sec. 5), and the greedy search with
latency savings measured on the GPU."""
import itertools

import numpy as np
import pytest

import workloads
from oracle.run import run_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io, vtog
    vt.lib()
    return vt, torch_io, pipelines, vtog, torch


def test_every_mixed_strategy_of_a_small_chain_gives_the_oracle_result(gpu):
    """Config 1's chain (permute, reshape, slice, concat): each subset of intermediates made
    virtual, the rest copied: all 2^4 strategies are bit-exact against the oracle."""
    vt, tio, pipelines, vtog, torch = gpu
    wl = workloads.c1_tiny_chain()
    ref = run_workload(wl)["out"].astype(np.float32)
    g = vtog.build_vtog(list(wl.chain), tuple(wl.sources), (), directions=("read",))
    tensors = sorted(g.by_tensor)
    assert len(tensors) == 4
    dw = tio.DeviceWorkload(wl)
    for r in range(len(tensors) + 1):
        for subset in itertools.combinations(tensors, r):
            chosen = {t: g.by_tensor[t][0] for t in subset}
            p = pipelines.StrategyPipeline(dw, chosen)
            assert len(p.copies) <= len(tensors) - len(subset)      # an intermediate nobody reads any more is not produced
            p.run()
            torch.cuda.synchronize()
            assert np.array_equal(p.out.cpu().numpy(), ref), subset


def test_strategy_extremes_match_the_two_fixed_paths(gpu):
    vt, tio, pipelines, vtog, torch = gpu
    wl = workloads.c2_decode_attention(seed=2, B=2, Hkv=2, G=4, S=257, D=128)
    dw = tio.DeviceWorkload(wl)
    g = vtog.build_vtog(list(wl.chain), tuple(wl.sources), (), directions=("read",))
    everything = {t: opps[0] for t, opps in g.by_tensor.items()}
    pv = pipelines.StrategyPipeline(dw, everything)
    pm = pipelines.StrategyPipeline(dw, {})
    assert pv.copies == [] and len(pm.copies) == len(g.by_tensor)
    ref = run_workload(wl)["out"]
    for p in (pv, pm):
        p.run()
        torch.cuda.synchronize()
        assert np.max(np.abs(tio.to_host_f64(p.out) - ref)) <= 2e-3


def test_greedy_with_measured_savings_virtualises_the_decode_chain(gpu):
    vt, tio, pipelines, vtog, torch = gpu
    wl = workloads.c2_decode_attention(seed=3, B=4, Hkv=4, G=4, S=1024, D=128)
    dw = tio.DeviceWorkload(wl)
    chosen, rep = pipelines.greedy_strategy(dw, iters=8)
    g = vtog.build_vtog(list(wl.chain), tuple(wl.sources), (), directions=("read",))
    assert vtog.is_points_to_graph(g, chosen)
    # the big copies (cache append, expand to 32 heads) must be gone and the saving must be real
    assert rep["saving_us"] > 0 and rep["chosen_us"] < 0.5 * rep["all_physical_us"], rep
    kv_chain = [t for t in g.by_tensor if t not in ("Q",)]
    assert sum(t in chosen for t in kv_chain) >= len(kv_chain) - 4, (sorted(chosen), rep)
    p = pipelines.StrategyPipeline(dw, chosen)
    p.run()
    torch.cuda.synchronize()
    assert np.max(np.abs(tio.to_host_f64(p.out) - run_workload(wl)["out"])) <= 2e-3


LEAN_CASES = [
    # name, workload, copies a stride-aware framework makes, appends it executes in place
    ("c1", lambda: workloads.c1_tiny_chain(), ["V"], 0),
    ("c2", lambda: workloads.c2_decode_attention(seed=4, B=2, Hkv=2, G=4, S=200, D=128, poison_last_slot=True), ["K", "V"], 2),
    ("c3", lambda: workloads.c3_oproj_gemm(seed=4, B=2, H=3, S=100, D=64, N=264), ["A"], 0),
    ("c4", lambda: workloads.c4_window_ln_linear(seed=4, B=2, R=14, win=7, C=128, N=384), ["T"], 0),
    ("c5", lambda: workloads.c5_moe_dispatch(seed=4, T=300, Hd=128, E=3, N=264), ["A0", "A1", "A2"], 0),
]


@pytest.mark.parametrize("name,make,copies,appends", LEAN_CASES, ids=[c[0] for c in LEAN_CASES])
def test_lean_materialized_path(gpu, name, make, copies, appends):
    """The lean comparison path (views stay views; only permute->reshape, expand->reshape, concat
    and index_select copy; a cache append is done in place) gives the oracle's result, and makes
    exactly the copies expected."""
    vt, tio, pipelines, vtog, torch = gpu
    wl = make()
    ref = run_workload(wl)["out"]
    stmts, chosen, scatters = pipelines.lean_plan(wl)
    assert sorted(s[0] for s in stmts if s[0] not in chosen) == sorted(copies)
    assert len(scatters) == appends
    dw = tio.DeviceWorkload(wl)            # the append writes into this copy of the sources
    p = pipelines.make_lean_pipeline(dw)
    assert len(p.copies) == len(copies) + appends
    for _ in range(2):                     # a second run finds the appended rows already in place
        p.run()
    torch.cuda.synchronize()
    out = p.out if p.out is not None else p.consumer.out
    if name == "c1":
        assert np.array_equal(out.cpu().numpy(), ref)
    else:
        got = tio.to_host_f64(out).reshape(ref.shape)
        assert (np.abs(got - ref) <= 1e-2 + 1e-2 * np.abs(ref)).all()
        # same consumer kernel as the virtual path: identical bits where both tile the work alike
        v = pipelines.make_pipeline(tio.DeviceWorkload(wl))
        v.run()
        torch.cuda.synchronize()
        if name in ("c3", "c4", "c5"):
            assert torch.equal(v.out, out)
    if name == "c2":
        # the new K/V rows now sit in slot S-1 of the caches (the poisoned slot was overwritten)
        S = 200
        qkv = tio.to_host_bits(dw.tensors["QKV"]).reshape(2, -1)
        kc = tio.to_host_bits(dw.tensors["Kcache"])
        assert np.array_equal(kc[:, :, S - 1, :].reshape(2, -1), qkv[:, 8 * 128:10 * 128])


def test_store_direction_choices_of_concat_inputs_are_lowered(gpu):
    """Config 1's Concat with its inputs made virtual tensors of its output (store direction,
    Sec. 4.4): each input is written straight into its columns of V, no buffer of its own, and the
    result is the oracle's, bit for bit, for every mix with read-direction choices upstream."""
    vt, tio, pipelines, vtog, torch = gpu
    wl = workloads.c1_tiny_chain(seed=5, a=3, b=8, c=40, lo=2, hi=20, ny=7)
    ref = run_workload(wl)["out"].astype(np.float32)
    g = vtog.build_vtog(list(wl.chain), tuple(wl.sources), ())
    store_t3 = next(o for o in g.by_tensor["t3"] if o.direction == "store" and o.targets == ("V",))
    read = {t: next(o for o in g.by_tensor[t] if o.direction == "read") for t in ("t1", "t2")}
    dw = tio.DeviceWorkload(wl)
    for upstream in ({}, {"t1": read["t1"]}, {"t2": read["t2"]}, dict(read)):
        chosen = dict(upstream)
        chosen["t3"] = store_t3
        assert vtog.is_points_to_graph(g, chosen)
        p = pipelines.StrategyPipeline(dw, chosen)
        assert "t3" not in p.bufs and "V" in p.bufs            # t3 lives inside V
        assert sum(isinstance(c[2], vt.Desc) for c in p.copies) == 2     # two stores into V: t3's part and Y's
        p.run()
        torch.cuda.synchronize()
        assert np.array_equal(p.out.cpu().numpy(), ref), sorted(chosen)
    # the append of the decode chain as a store: the new K/V row is written into the concatenated tensor
    wl = workloads.c2_decode_attention(seed=6, B=2, Hkv=2, G=4, S=130, D=128)
    g = vtog.build_vtog(list(wl.chain), tuple(wl.sources), ())
    chosen = {t: next(o for o in g.by_tensor[t] if o.direction == "read") for t in g.by_tensor if t not in ("kn", "vn", "kf", "vf")}
    for t, c in (("kn", "kf"), ("vn", "vf")):
        chosen[t] = next(o for o in g.by_tensor[t] if o.direction == "store" and o.targets == (c,))
    assert vtog.is_points_to_graph(g, chosen)
    p = pipelines.StrategyPipeline(tio.DeviceWorkload(wl), chosen)
    p.run()
    torch.cuda.synchronize()
    assert np.max(np.abs(tio.to_host_f64(p.out) - run_workload(wl)["out"])) <= 2e-3


BIJECTIVE_STORES = [
    # workload, tensor stored into the output of a bijective operator, tolerance (None: bit-exact)
    ("c1", lambda: workloads.c1_tiny_chain(seed=7, a=3, b=8, c=40, lo=2, hi=20, ny=7), ["t1"], None),
    ("c3", lambda: workloads.c3_oproj_gemm(seed=7, B=2, H=3, S=100, D=64, N=264), ["o1"], 1e-2),
    ("c4 permute", lambda: workloads.c4_window_ln_linear(seed=7, B=2, R=14, win=7, C=128, N=384), ["x1"], 1e-2),
    ("c4 reshape", lambda: workloads.c4_window_ln_linear(seed=7, B=2, R=14, win=7, C=128, N=384), ["x2"], 1e-2),
    ("c4 both", lambda: workloads.c4_window_ln_linear(seed=7, B=2, R=14, win=7, C=128, N=384), ["x1", "x2"], 1e-2),
]


@pytest.mark.parametrize("name,make,tensors,tol", BIJECTIVE_STORES, ids=[c[0] for c in BIJECTIVE_STORES])
def test_store_direction_through_reshape_and_permute(gpu, name, make, tensors, tol):
    """The input of a Reshape or Permute made a virtual tensor of the operator's output (store
    direction, Sec. 4.4): what produces the input is written through the inverse view of the output,
    the operator itself is never executed, and the consumer's result is the oracle's."""
    vt, tio, pipelines, vtog, torch = gpu
    wl = make()
    ref = run_workload(wl)["out"]
    g = vtog.build_vtog(list(wl.chain), tuple(wl.sources), ())
    chosen = {t: next(o for o in g.by_tensor[t] if o.direction == "store") for t in tensors}
    assert vtog.is_points_to_graph(g, chosen)
    p = pipelines.StrategyPipeline(tio.DeviceWorkload(wl), chosen)
    for t in tensors:
        assert t not in p.bufs                                    # lives inside the operator's output
    assert sum(isinstance(c[2], vt.Desc) for c in p.copies) >= 1  # written through a map
    p.run()
    torch.cuda.synchronize()
    out = p.out if p.out is not None else p.consumer.out
    if tol is None:
        assert np.array_equal(out.cpu().numpy(), ref.astype(np.float32))
    else:
        got = tio.to_host_f64(out).reshape(ref.shape)
        assert (np.abs(got - ref) <= tol + tol * np.abs(ref)).all()


def test_one_output_of_a_split_gives_its_input_no_store_bundle(gpu):
    """The executable chains name one output of a Split per statement.  The Split's input cannot be
    stitched from outputs that are not all there, so the opportunity graph offers it no
    store-direction bundle (a whole Split, all outputs in one statement, does: tests/test_vtog.py);
    the read-direction choices run."""
    vt, tio, pipelines, vtog, torch = gpu
    rng = np.random.default_rng(0)
    src = {"X": rng.standard_normal((4, 6)).astype(np.float32), "Z": rng.standard_normal((2, 4)).astype(np.float32)}
    chain = [("t0", "permute", ("X",), {"perm": (1, 0)}),
             ("a", "split", ("t0",), {"dim": 0, "sizes": (2, 4), "output": 0})]
    wl = workloads.Workload("split_read", "f32", src, chain, {"kind": "add_rowsum", "x": "a", "y": "Z"})
    g = vtog.build_vtog(list(wl.chain), tuple(wl.sources), ())
    assert [o.direction for o in g.by_tensor["t0"]] == ["read"] and [o.direction for o in g.by_tensor["a"]] == ["read"]
    whole = vtog.build_vtog([chain[0], (("a", "b"), "split", ("t0",), {"dim": 0, "sizes": (2, 4)})], ("X",), ())
    stores = [o for o in whole.by_tensor["t0"] if o.direction == "store"]
    assert [o.targets for o in stores] == [("a", "b")]
    with pytest.raises(vt.VtError):          # a legal bundle that this lowering does not execute: it says so
        pipelines.StrategyPipeline(tio.DeviceWorkload(wl), {"t0": stores[0]},
                                   statements=[chain[0], (("a", "b"), "split", ("t0",), {"dim": 0, "sizes": (2, 4)})])
    chosen = {t: g.by_tensor[t][0] for t in ("t0", "a")}
    p = pipelines.StrategyPipeline(tio.DeviceWorkload(wl), chosen)
    p.run()
    torch.cuda.synchronize()
    assert np.array_equal(p.out.cpu().numpy(), run_workload(wl)["out"].astype(np.float32))
