"""The hot path captured into HIP graphs (how bench.py launches it): every replay must give the
bits of the same launches made one by one, also after the inputs changed between replays and with
ordinary launches and synchronizations in between."""
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


def capture(torch, fns):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for fn in fns:
            fn(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for fn in fns:
            fn(side)
    torch.cuda.synchronize()
    return g


def test_decode_segment_replays_equal_eager_launches(gpu):
    """Projection with the producer-side store, then attention over the caches it wrote (two
    kernels with split merges on workspaces whose counters must return to zero), as one graph."""
    vt, tio, pipelines, torch = gpu
    st1, st2 = workloads.decode_segment(seed=11, B=2, hidden=256, Hkv=2, G=4, D=128, cap=300, pos=299)
    seg = pipelines.DecodeSegment(st1, st2)
    r1 = run_workload(st1)
    st2.sources = {k: r1["stored"][k] for k in st2.sources}
    ref = run_workload(st2)["out"]
    seg.run()
    torch.cuda.synchronize()
    eager = seg.out.clone()
    assert np.max(np.abs(tio.to_host_f64(eager) - ref)) <= 2e-3
    g = capture(torch, [lambda s: seg.run(stream=s)])
    x = seg.dw1.tensors["X"]
    x0 = x.clone()
    for rep in range(4):
        if rep % 2:                       # other activations: the graph reads the same buffers
            x.copy_(torch.flip(x0, dims=(0,)))
        else:
            x.copy_(x0)
        seg.out.zero_()
        g.replay()
        torch.cuda.synchronize()
        got = seg.out.clone()
        seg.out.zero_()
        seg.run()                         # the program's own eager launch between the replays
        torch.cuda.synchronize()
        assert torch.equal(got, seg.out), rep
        if rep % 2 == 0:
            assert torch.equal(got, eager), rep


def test_static_workspace_attention_in_a_graph(gpu):
    """The entry point without allocation queues a fill kernel and the attention kernel: both are
    captured, and replays on changing inputs equal vt_decode_attn on the same inputs."""
    vt, tio, pipelines, torch = gpu
    wl = workloads.c2_decode_attention(seed=12, B=2, Hkv=2, G=4, S=777, D=128)
    dw = tio.DeviceWorkload(wl)
    p = pipelines.DecodeAttention(dw, want_lse=False)
    out_s = torch.zeros_like(p.out)
    g = capture(torch, [lambda s: vt.vt_decode_attn_static(p.q, p.k, p.v, p.scale, out_s, stream=s)])
    qkv = dw.tensors["QKV"]
    q0 = qkv.clone()
    for rep in range(3):
        qkv.copy_(torch.roll(q0, shifts=rep, dims=0))
        out_s.zero_()
        g.replay()
        p.run()                           # eager, ordinary workspace, same stream order
        torch.cuda.synchronize()
        assert torch.equal(out_s, p.out), rep
    qkv.copy_(q0)
    g.replay()
    torch.cuda.synchronize()
    assert np.max(np.abs(tio.to_host_f64(out_s) - run_workload(wl)["out"])) <= 2e-3


def test_every_benchmark_chain_kind_replays_bitwise(gpu):
    """One small workload per consumer kernel, virtual and lean-materialized launches in one
    graph, replayed three times against the launches made one by one."""
    vt, tio, pipelines, torch = gpu
    makes = [
        lambda: workloads.c1_tiny_chain(),
        lambda: workloads.c3_oproj_gemm(seed=3, B=2, H=3, S=100, D=64, N=264),
        lambda: workloads.c4_window_ln_linear(seed=3, B=2, R=14, win=7, C=128, N=384),
        lambda: workloads.c5_moe_dispatch(seed=3, T=300, Hd=128, E=3, N=264),
        lambda: workloads.moe_combine(seed=3, T=257, E=4, N=512),
        lambda: workloads.rowsum_chain_large(seed=3, A=4, B=96, C0=64, ny=48),
    ]
    for make in makes:
        wl = make()
        v = pipelines.make_pipeline(tio.DeviceWorkload(wl))
        m = pipelines.make_lean_pipeline(tio.DeviceWorkload(wl))
        outs = lambda: [x.out if x.out is not None else x.consumer.out for x in (v, m)]   # noqa: E731
        v.run()
        m.run()
        torch.cuda.synchronize()
        want = [o.clone() for o in outs()]
        g = capture(torch, [lambda s: v.run(stream=s), lambda s: m.run(stream=s)])
        for rep in range(3):
            for o in outs():
                o.zero_()
            g.replay()
            torch.cuda.synchronize()
            for o, w in zip(outs(), want):
                assert torch.equal(o, w), (wl.name, rep)
            v.run()                       # eager work between the replays
            torch.cuda.synchronize()
