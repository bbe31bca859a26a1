"""Degenerate and extreme shapes through the C ABI: empty tensors, a single key, one row, one
column block, group size 16."""
import numpy as np
import pytest

import workloads
from oracle import consumers, dm_ops
from oracle.run import run_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io
    vt.lib()
    return vt, torch_io, pipelines, torch


def test_empty_tensors_are_refused_when_the_descriptor_is_built(gpu):
    """A tensor without elements never reaches a kernel: vt_build reports VT_ERR_SHAPE for an
    empty source and for a slice that selects nothing."""
    vt, tio, pipelines, torch = gpu
    keep = torch.full((4,), 7.0, dtype=torch.float32, device="cuda:0")
    with pytest.raises(vt.VtError) as ei:
        vt.build_chain([], {"X": ((0, 8), "f32", keep.data_ptr())}, "X")
    assert ei.value.code == vt.ERR_SHAPE
    with pytest.raises(vt.VtError) as ei:
        vt.build_chain([("s", "slice", ("X",), {"dim": 0, "start": 2, "stop": 2})], {"X": ((4,), "f32", keep.data_ptr())}, "s")
    assert ei.value.code in (vt.ERR_SHAPE, vt.ERR_RANGE)
    torch.cuda.synchronize()
    assert torch.equal(keep, torch.full((4,), 7.0, device="cuda:0"))


def test_attention_over_two_keys(gpu):
    """The shortest context the decode chain can describe: one cached row and the fresh one."""
    vt, tio, pipelines, torch = gpu
    wl = workloads.c2_decode_attention(seed=1, B=2, Hkv=2, G=4, S=2, D=128)
    res = pipelines.run_decode_attention(tio.DeviceWorkload(wl))
    ref = run_workload(wl)
    assert np.max(np.abs(tio.to_host_f64(res["out"]) - ref["out"])) <= 1e-2
    # a convex combination of the two value rows: between them, element by element
    v = consumers.decode(dm_ops.run_chain(wl.chain, wl.sources)["V"], "bf16")
    got = tio.to_host_f64(res["out"])
    assert (got <= v.max(axis=2) + 1e-2).all() and (got >= v.min(axis=2) - 1e-2).all()


@pytest.mark.parametrize("G,S", [(16, 70), (1, 33), (8, 4097)])
def test_attention_group_sizes_and_ragged_contexts(gpu, G, S):
    vt, tio, pipelines, torch = gpu
    wl = workloads.c2_decode_attention(seed=2, B=1, Hkv=2, G=G, S=S, D=128)
    res = pipelines.run_decode_attention(tio.DeviceWorkload(wl))
    ref = run_workload(wl)
    assert np.max(np.abs(tio.to_host_f64(res["out"]) - ref["out"])) <= 3e-3
    assert np.max(np.abs(tio.to_host_f64(res["lse"]) - ref["lse"])) <= 1e-3


def test_gemm_one_row_one_column_block(gpu):
    vt, tio, pipelines, torch = gpu
    wl = workloads.c3_oproj_gemm(seed=3, B=1, H=1, S=1, D=64, N=8)      # M = 1, K = 64, N = 8
    p = pipelines.Gemm(tio.DeviceWorkload(wl))
    p.run()
    torch.cuda.synchronize()
    ref = run_workload(wl)["out"]
    assert np.max(np.abs(tio.to_host_f64(p.out) - ref)) <= 1e-2 + 1e-2 * np.abs(ref).max()


def test_store_gemm_minimal(gpu):
    vt, tio, pipelines, torch = gpu
    wl = workloads.qkv_proj_store(seed=4, B=1, hidden=8, Hq=1, Hkv=1, D=8, cap=2, pos=1, T=1)   # M = 1, K = 8, N = 24
    ref = run_workload(wl)
    dw = tio.DeviceWorkload(wl)
    pipelines.GemmStore(dw).run()
    torch.cuda.synchronize()
    for name, want in ref["stored"].items():
        got = consumers.decode(tio.to_host_bits(dw.tensors[name]), "bf16")
        assert np.max(np.abs(got - consumers.decode(want, "bf16"))) <= 1e-2, name
