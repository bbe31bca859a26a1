"""GPU parity of the window-partition -> LayerNorm -> linear chain (fp16; LayerNorm fused into the
GEMM's load stage, and the unfused LayerNorm kernel + GEMM) against the CPU oracle.
Tolerance |gpu - oracle| <= 1e-2 + 1e-2 |oracle| (the benchmark states none for fp16: the bf16
bar is used; observed errors are ~1e-3, see the asserts on the maximum)."""
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
    from paper_2604_09558_amd import pipelines, torch_io
    vt.lib()
    return vt, torch_io, pipelines, torch


def check(got, ref, atol=1e-2, rtol=1e-2):
    err = np.abs(got - ref)
    bad = err > atol + rtol * np.abs(ref)
    assert not bad.any(), "max abs err %.3e at %s" % (err.max(), np.unravel_index(err.argmax(), err.shape))
    return err.max()


CASES = [
    # B, R, win, C, N, dtype
    (2, 14, 7, 128, 384, "f16"),       # 8 windows of 49 tokens: 392 rows (6 blocks + a ragged one)
    (1, 6, 3, 128, 264, "f16"),        # N not a multiple of 128: masked columns
    (3, 8, 4, 64, 128, "f16"),         # K = 64, one column block per wave
    (2, 14, 7, 128, 384, "bf16"),
    (1, 21, 7, 64, 200, "bf16"),
]


@pytest.mark.parametrize("B,R,win,C,N,dtype", CASES)
def test_c4_fused_small(gpu, B, R, win, C, N, dtype):
    vt, tio, pipelines, torch = gpu
    wl = workloads.c4_window_ln_linear(seed=1, B=B, R=R, win=win, C=C, N=N, dtype=dtype)
    ref = run_workload(wl)["out"]
    p = pipelines.Gemm(tio.DeviceWorkload(wl), fused=True)
    p.run()
    torch.cuda.synchronize()
    got = tio.to_host_f64(p.out).reshape(ref.shape)
    check(got, ref)


def test_c4_unfused_and_materialized_agree(gpu):
    vt, tio, pipelines, torch = gpu
    wl = workloads.c4_window_ln_linear(seed=2, B=2, R=14, win=7, C=128, N=384)
    ref = run_workload(wl)["out"]
    dw = tio.DeviceWorkload(wl)
    outs = {}
    for name, kw in (("fused", dict(fused=True)), ("unfused", dict(fused=False)),
                     ("mat_fused", dict(fused=True, materialized=True))):
        p = pipelines.Gemm(dw, **kw)
        p.run()
        torch.cuda.synchronize()
        outs[name] = tio.to_host_f64(p.out).reshape(ref.shape)
        check(outs[name], ref)
    # same kernel on dense copies of the intermediates: identical bits
    assert np.array_equal(outs["fused"], outs["mat_fused"])


def test_c4_full_size(gpu):
    """Config 4 at the benchmark's size: every output compared."""
    vt, tio, pipelines, torch = gpu
    wl = workloads.c4_window_ln_linear()
    ref = run_workload(wl)["out"]
    p = pipelines.Gemm(tio.DeviceWorkload(wl), fused=True)
    p.run()
    torch.cuda.synchronize()
    got = tio.to_host_f64(p.out).reshape(ref.shape)
    mx = check(got, ref)
    assert mx <= 4e-3, mx      # outputs ~N(0, 0.23): fp16 rounding of LN (2^-11 rel) and of the result


def test_constant_rows_give_zero(gpu):
    """LayerNorm of a constant row is zero, so the product is zero (no NaN from 0 * rsqrt(eps))."""
    vt, tio, pipelines, torch = gpu
    wl = workloads.c4_window_ln_linear(seed=3, B=1, R=6, win=3, C=128, N=128)
    wl.sources["X"][:] = np.float16(3.25)
    p = pipelines.Gemm(tio.DeviceWorkload(wl), fused=True)
    p.run()
    torch.cuda.synchronize()
    assert np.all(tio.to_host_f64(p.out) == 0.0)


def test_c4_one_full_round_plus_a_partial_one_and_f32_output(gpu):
    """21 952 rows on 256 compute units: one round of full blocks, then 87 workgroups with one more
    block (the last of them ragged); also the fp32-output path of the fused kernel."""
    vt, tio, pipelines, torch = gpu
    wl = workloads.c4_window_ln_linear(seed=4, B=7, R=56, win=7, C=128, N=384)
    ref = run_workload(wl)["out"]
    p = pipelines.Gemm(tio.DeviceWorkload(wl), fused=True)
    p.run()
    torch.cuda.synchronize()
    check(tio.to_host_f64(p.out).reshape(ref.shape), ref)
    out32 = torch.empty((ref.shape[0] * ref.shape[1], ref.shape[2]), dtype=torch.float32, device="cuda:0")
    vt.vt_gemm(p.A, p.B, [out32.data_ptr()], "f32", vt.GEMM_LAYERNORM, p.eps)
    torch.cuda.synchronize()
    # no final rounding to fp16: only the fp16 rounding of the normalised rows remains
    check(out32.cpu().numpy().astype(np.float64).reshape(ref.shape), ref, atol=2e-3, rtol=2e-3)


@pytest.mark.parametrize("B,R,win,C,N,dtype", [(1, 6, 3, 96, 200, "f16"), (1, 4, 2, 256, 520, "bf16"), (2, 6, 3, 40, 24, "f16")])
def test_shapes_outside_the_fused_kernel_run_on_the_generic_one(gpu, B, R, win, C, N, dtype):
    """Feature sizes other than 64 / 128 and more than 384 outputs: the LayerNorm prologue runs in
    the generic kernel (whole map per element), same values to the same tolerance."""
    vt, tio, pipelines, torch = gpu
    wl = workloads.c4_window_ln_linear(seed=5, B=B, R=R, win=win, C=C, N=N, dtype=dtype)
    ref = run_workload(wl)["out"]
    p = pipelines.Gemm(tio.DeviceWorkload(wl), fused=True)
    p.run()
    torch.cuda.synchronize()
    check(tio.to_host_f64(p.out).reshape(ref.shape), ref)
