"""The attention entry point that allocates nothing (vt_decode_attn_static: its workspace is a
fixed array inside the library's device memory) against vt_decode_attn on a caller's workspace:
same kernel, same split, so the bits must agree; and both against the CPU oracle to the
benchmark's bar.  Two calls in a row share the array, the second on a smaller problem."""
import numpy as np
import pytest

import workloads
from oracle.run import run_workload

pytestmark = pytest.mark.gpu


def _both(vt, tio, pipelines, torch, wl, n_splits=0):
    dw = tio.DeviceWorkload(wl)
    p = pipelines.DecodeAttention(dw, n_splits=n_splits)
    p.run()
    torch.cuda.synchronize()
    want_out, want_lse = tio.to_host_bits(p.out), p.lse.cpu().numpy().copy()
    out = torch.full_like(p.out, float("nan"))
    lse = torch.full_like(p.lse, float("nan"))
    vt.vt_decode_attn_static(p.q, p.k, p.v, p.scale, out, n_splits=n_splits, lse=lse)
    torch.cuda.synchronize()
    return want_out, want_lse, tio.to_host_bits(out), lse.cpu().numpy(), tio.to_host_f64(out)


def test_static_workspace_two_calls_second_smaller():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io as tio
    assert vt.vt_decode_attn_static_capacity() == 4 << 20
    cases = [dict(seed=11, B=4, Hkv=4, G=4, S=1500, D=128),     # several splits, ragged last tile
             dict(seed=12, B=2, Hkv=2, G=4, S=300, D=128)]      # smaller: fewer units, fewer splits
    for kw in cases:
        wl = workloads.c2_decode_attention(**kw)
        ref = run_workload(wl)
        want_out, want_lse, got_out, got_lse, got_f64 = _both(vt, tio, pipelines, torch, wl)
        assert np.array_equal(got_out, want_out), kw
        assert np.array_equal(got_lse.view(np.uint32), want_lse.view(np.uint32)), kw
        err = np.abs(got_f64 - ref["out"])
        assert (err <= 1e-2 + 1e-2 * np.abs(ref["out"])).all(), (kw, err.max())
        assert np.max(np.abs(got_lse - ref["lse"])) <= 2e-3


def test_static_workspace_rejects_what_does_not_fit():
    import torch
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io as tio
    # 16 x 32 heads x 64 splits x 130 floats = 17 MB of partial results: beyond the 4 MiB array
    wl = workloads.c2_decode_attention(seed=13, B=16, Hkv=8, G=4, S=2048, D=128)
    dw = tio.DeviceWorkload(wl)
    p = pipelines.DecodeAttention(dw, n_splits=64)
    assert p.ws_bytes > vt.vt_decode_attn_static_capacity()
    with pytest.raises(vt.VtError) as ei:
        vt.vt_decode_attn_static(p.q, p.k, p.v, p.scale, p.out, n_splits=64)
    assert ei.value.code == vt.ERR_INVALID_ARG and "workspace too small" in str(ei.value)
    torch.cuda.synchronize()
