"""GPU parity of the mixture-of-experts combine (weighted sum of two rows gathered through routing
tables) against the oracle: one rounding of an fp32 result to bf16/f16."""
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


def check(got, ref, rel):
    err = np.abs(got - ref)
    assert (err <= rel * np.abs(ref) + 1e-6).all(), err.max()


@pytest.mark.parametrize("T,E,N,dtype", [(300, 4, 264, "bf16"), (64, 8, 8, "f16"), (1000, 8, 1000, "bf16"), (50, 3, 20, "f16")])
def test_moe_combine_small(gpu, T, E, N, dtype):
    vt, tio, pipelines, torch = gpu
    wl = workloads.moe_combine(seed=1, T=T, E=E, N=N, dtype=dtype)     # N = 20: rows are not 16-byte multiples -> generic path
    ref = run_workload(wl)["out"]
    for materialized in (False, True):
        p = pipelines.WeightedSum(tio.DeviceWorkload(wl), materialized)
        p.run()
        torch.cuda.synchronize()
        # fp32 product-sum (3 roundings of 2^-24) then one rounding to the storage type
        check(tio.to_host_f64(p.out), ref, 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11)


def test_moe_combine_virtual_equals_materialized_bitwise_and_mid_size(gpu):
    vt, tio, pipelines, torch = gpu
    wl = workloads.moe_combine(seed=2, T=4096, E=8, N=2048)
    a = pipelines.WeightedSum(tio.DeviceWorkload(wl))
    b = pipelines.WeightedSum(tio.DeviceWorkload(wl), materialized=True)
    a.run()
    b.run()
    torch.cuda.synchronize()
    assert torch.equal(a.out, b.out)
    check(tio.to_host_f64(a.out), run_workload(wl)["out"], 2.0 ** -8)


def test_moe_combine_full_size_every_output(gpu):
    """The combine at the benchmarked size (16384 tokens x 14336 columns), every output; the oracle
    gathers both operands as dense copies and mixes them in float64, in row blocks to bound memory."""
    vt, tio, pipelines, torch = gpu
    wl = workloads.moe_combine()
    p = pipelines.WeightedSum(tio.DeviceWorkload(wl))
    p.run()
    torch.cuda.synchronize()
    env = dm_ops.run_chain(wl.chain, wl.sources, wl.index_tables, keep={"x", "y"})
    w = wl.consumer["weights"]
    assert env["x"].shape == (16384, 14336)
    for r in range(0, 16384, 2048):
        ref = consumers.weighted_sum(consumers.decode(env["x"][r:r + 2048], "bf16"),
                                     consumers.decode(env["y"][r:r + 2048], "bf16"), w[r:r + 2048])
        check(tio.to_host_f64(p.out[r:r + 2048]), ref, 2.0 ** -8)
