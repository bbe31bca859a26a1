#!/usr/bin/env python3
"""Benchmark of the virtual-tensor hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: the consumer
kernel reading its operands through the descriptors (virtual path).  The default workload is
the Llama-3-8B-shaped decode segment (config 2 of the benchmark spec): fused QKV output + KV cache
-> GQA flash-decoding, bf16, batch 8, context 4096.

Inputs are resident in HBM before the timed region.  To keep the 256 MB Infinity Cache from
serving the 134 MB working set, the steps rotate over several independent copies of the
inputs (more than 1 GB in total), so every step streams its K/V from HBM.

Prints one JSON line (see the fields at the bottom).  `--gpus N` with N > 1 is refused: this
build is single-GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X published dense bf16/fp16 matrix peak


def algorithmic_bytes_c2(B, Hkv, G, S, D, n_splits, esz=2):
    """Bytes the method itself must move for one decode-attention step (kernel
    table): K and V once (un-expanded), the fused QKV row, the output, and the split-K partial
    results written once and read once."""
    Hq = Hkv * G
    kv = 2 * B * Hkv * S * D * esz
    qkv = B * (Hq + 2 * Hkv) * D * esz
    out = B * Hq * D * esz
    ws = 2 * B * Hq * n_splits * (D + 2) * 4
    return kv + qkv + out + ws


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--copies", type=int, default=8, help="independent input copies the steps rotate over")
    ap.add_argument("--no-graph", action="store_true", help="launch every step from Python instead of replaying a HIP graph")
    ap.add_argument("--no-materialized", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--n-splits", type=int, default=0, help="context splits of the attention kernel (0 = library's choice)")
    ap.add_argument("--context", type=int, default=4096, help="context length (the benchmark's is 4096; others are for tuning)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 128 MiB -> 128 MiB copy kernel 20 times (reference point for HBM byte counters)")
    ap.add_argument("--extra", default="", help="comma list of further chains to time (c1,c3,c4,c5,qkv_store,decode_segment,paged,moe_combine)")
    return ap.parse_args()


def time_steps(torch, step_fns, steps, warmup, use_graph):
    """Runs warmup + exactly `steps` calls of step_fns[k % R] on the current stream, bracketed by
    synchronize on both sides, and by two HIP events on that stream.  With use_graph the R
    step functions are captured once into one HIP graph (R launches per replay); steps that
    do not fill a whole replay are launched eagerly.  Returns (wall ms per step, event ms per
    step)."""
    R = len(step_fns)
    stream = torch.cuda.current_stream()
    graph = None
    if use_graph and steps >= R:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            for fn in step_fns:
                fn(side)            # warm the code path on the capture stream
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for fn in step_fns:
                fn(side)
        torch.cuda.synchronize()

    def run(n):
        k = 0
        if graph is not None:
            while k + R <= n:
                graph.replay()
                k += R
        while k < n:
            step_fns[k % R](stream)
            k += 1

    run(warmup)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    run(steps)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def cpu_baseline_c2(wl, alg_bytes):
    """The oracle as it stands on the host cores: one full pass (materialize every op, then
    fp64 attention) over the same workload."""
    import psutil
    from oracle.run import run_workload
    proc = psutil.Process()
    c0 = proc.cpu_times()
    t0 = time.perf_counter()
    run_workload(wl)
    dt = time.perf_counter() - t0
    c1 = proc.cpu_times()
    cpu = (c1.user - c0.user) + (c1.system - c0.system)
    return {"value": alg_bytes / dt / 1e9, "unit": "GB/s", "cores": max(1, int(round(cpu / dt))), "kind": "oracle",
            "sample": "one full pass of config 2 (B=8, context 4096): %.2f s wall" % dt, "seconds": dt}


def chain_stats(torch, name, steps, a_no_graph=False):
    """Virtual and materialized (every operator an explicit copy kernel) timings of one of the
    other benchmark chains; inputs rotate over enough copies to defeat the Infinity Cache where
    the working set is small."""
    import workloads
    from paper_2604_09558_amd import pipelines
    from paper_2604_09558_amd import torch_io as tio
    if name == "decode_segment":
        # projection with a producer-side store + attention on the caches it wrote (Sec. 3.1)
        mk = lambda p: (lambda stream: p.run(stream))      # noqa: E731
        segs = [pipelines.DecodeSegment(*workloads.decode_segment(seed=s)) for s in range(4)]
        torch.cuda.synchronize()
        v_wall, v_ev = time_steps(torch, [mk(p) for p in segs], steps, max(2, steps // 10), True)
        M, N, K = segs[0].store.shape
        B, Hq, S, D = segs[0].attn.k.shape
        alg = (K * N + M * K + M * N) * 2 + 2 * B * (Hq // 4) * S * D * 2 + 2 * B * Hq * D * 2
        out = {"virtual_us": round(v_ev * 1e3, 2), "algorithmic_bytes": int(alg),
               "hbm_pct_of_peak": round(100.0 * alg / (v_ev * 1e-3) / 1e9 / HBM_PEAK_GBS, 1)}
        del segs
        torch.cuda.empty_cache()
        mat = pipelines.DecodeSegment(*workloads.decode_segment(seed=0), materialized=True)
        torch.cuda.synchronize()
        m_wall, m_ev = time_steps(torch, [mk(mat)], max(5, steps // 8), 2, False)
        out["materialized_full_us"] = round(m_ev * 1e3, 2)
        out["speedup_vs_materialized_full"] = round(m_ev / v_ev, 2)
        out["intermediate_bytes_saved"] = int(mat.attn.mat.bytes_written + M * N * 2)
        return out
    if name == "moe_combine":
        # the combine after config 5: two gathered rows per token, mixed with the routing weights
        mk = lambda p: (lambda stream: p.run(stream))      # noqa: E731
        dw = tio.DeviceWorkload(workloads.moe_combine())
        pv = pipelines.WeightedSum(dw)
        torch.cuda.synchronize()
        v_wall, v_ev = time_steps(torch, [mk(pv)], steps, max(2, steps // 10), False)
        R, C = pv.x.shape
        alg = 3 * R * C * 2 + R * 16
        out = {"virtual_us": round(v_ev * 1e3, 2), "algorithmic_bytes": int(alg),
               "hbm_pct_of_peak": round(100.0 * alg / (v_ev * 1e-3) / 1e9 / HBM_PEAK_GBS, 1)}
        pm = pipelines.WeightedSum(dw, materialized=True)
        torch.cuda.synchronize()
        m_wall, m_ev = time_steps(torch, [mk(pm)], max(5, steps // 4), 2, False)
        out["materialized_full_us"] = round(m_ev * 1e3, 2)
        out["speedup_vs_materialized_full"] = round(m_ev / v_ev, 2)
        out["intermediate_bytes_saved"] = int(pm.mat.bytes_written)
        return out
    if name == "paged":
        # config 2's attention over a paged KV cache (pages of 128 rows picked through a block table)
        mk = lambda p: (lambda stream: p.run(stream))      # noqa: E731
        dws = [tio.DeviceWorkload(workloads.paged_decode_attention(seed=s)) for s in range(4)]
        ps = [pipelines.DecodeAttention(dw, want_lse=False) for dw in dws]
        torch.cuda.synchronize()
        v_wall, v_ev = time_steps(torch, [mk(p) for p in ps], steps, max(2, steps // 10), True)
        B, Hq, S, D = ps[0].k.shape
        alg = 2 * B * (Hq // 4) * S * D * 2 + 2 * B * Hq * D * 2
        out = {"virtual_us": round(v_ev * 1e3, 2), "algorithmic_bytes": int(alg),
               "hbm_pct_of_peak": round(100.0 * alg / (v_ev * 1e-3) / 1e9 / HBM_PEAK_GBS, 1)}
        del ps, dws
        torch.cuda.empty_cache()
        mat = pipelines.DecodeAttention(tio.DeviceWorkload(workloads.paged_decode_attention(seed=0)), materialized=True, want_lse=False)
        torch.cuda.synchronize()
        m_wall, m_ev = time_steps(torch, [mk(mat)], max(5, steps // 8), 2, False)
        out["materialized_full_us"] = round(m_ev * 1e3, 2)
        out["speedup_vs_materialized_full"] = round(m_ev / v_ev, 2)
        out["intermediate_bytes_saved"] = int(mat.mat.bytes_written)
        return out
    copies = {"c1": 1, "c3": 3, "c4": 6, "c5": 1, "qkv_store": 6}[name]
    wls = [workloads.CONFIGS[name](seed=s) for s in range(copies)]
    dws = [tio.DeviceWorkload(w) for w in wls]
    virt = [pipelines.make_pipeline(dw) for dw in dws]
    torch.cuda.synchronize()
    mk = lambda p: (lambda stream: p.run(stream))      # noqa: E731
    n = steps
    # short kernels are launched from one HIP graph, like the main line (a Python launch costs more than they run)
    graph_ok = name in ("c1", "c4", "qkv_store") and not a_no_graph
    rep = 16 // len(virt) + 1 if graph_ok else 1     # a graph replay should hold a good number of launches
    v_wall, v_ev = time_steps(torch, [mk(p) for p in virt] * rep, n, max(2, n // 10), graph_ok)
    out = {"virtual_us": round(v_ev * 1e3, 2)}
    p0 = virt[0]
    if name in ("c3", "c5", "c4"):
        rows, N, K = sum(p0.rows), p0.N, p0.A[0].shape[-1]
        flops = 2.0 * rows * N * K
        out["tflops"] = round(flops / (v_ev * 1e-3) / 1e12, 1)
        out["mfma_pct_of_peak"] = round(100.0 * flops / (v_ev * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 1)
        esz = 2
        a_bytes = rows * K * esz if name != "c5" else dws[0].tensors["tokens"].numel() * esz
        alg = a_bytes + len(p0.B) * K * N * esz + rows * N * esz
        out["algorithmic_bytes"] = int(alg)
        out["hbm_pct_of_peak"] = round(100.0 * alg / (v_ev * 1e-3) / 1e9 / HBM_PEAK_GBS, 1)
    if name == "qkv_store":
        # the weight is read once; the rows, the outputs and the K-slice partial sums are small
        M, N, K = p0.shape
        alg = (K * N + M * K + M * N) * 2
        out["algorithmic_bytes"] = int(alg)
        out["hbm_pct_of_peak"] = round(100.0 * alg / (v_ev * 1e-3) / 1e9 / HBM_PEAK_GBS, 1)
        mats = [pipelines.make_pipeline(dw, materialized=True) for dw in dws]
        torch.cuda.synchronize()
        m_wall, m_ev = time_steps(torch, [mk(p) for p in mats] * (1 if a_no_graph else 3), n, max(2, n // 10), not a_no_graph)
        out["materialized_full_us"] = round(m_ev * 1e3, 2)
        out["speedup_vs_materialized_full"] = round(m_ev / v_ev, 3)
        out["intermediate_bytes_saved"] = int(M * N * 2)
        return out
    mat = pipelines.make_pipeline(dws[0], materialized=True)
    torch.cuda.synchronize()
    m_graph = name == "c1" and not a_no_graph
    m_wall, m_ev = time_steps(torch, [mk(mat)] * (16 if m_graph else 1), max(16 if m_graph else 3, n // 4), 2, m_graph)
    out["materialized_full_us"] = round(m_ev * 1e3, 2)
    out["speedup_vs_materialized_full"] = round(m_ev / v_ev, 3)
    out["intermediate_bytes_saved"] = int(mat.mat.bytes_written)
    if name == "c4":
        unf = pipelines.Gemm(dws[0], fused=False)
        u_wall, u_ev = time_steps(torch, [mk(unf)], n, 2, False)
        out["virtual_unfused_us"] = round(u_ev * 1e3, 2)
    return out


def main():
    a = parse()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (one MI355X); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2604_09558_amd as vt
    import workloads
    from paper_2604_09558_amd import pipelines
    from paper_2604_09558_amd import torch_io as tio

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    vt.lib()
    torch.cuda.set_device(0)
    if a.calibrate_copy:
        # a plain copy of known size: reads 134217728 B and writes 134217728 B per launch
        n = 64 * 1024 * 1024
        srcs = [torch.ones(n, dtype=torch.bfloat16, device="cuda:0") for _ in range(4)]
        dst = torch.empty(n, dtype=torch.bfloat16, device="cuda:0")
        descs = [vt.build_chain([], {"X": ((n,), "bf16", t.data_ptr())}, "X") for t in srcs]
        for k in range(20):
            vt.vt_materialize(descs[k % 4], dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "k_materialize copies 134217728 B -> 134217728 B", "launches": 20}))
        return
    B, Hkv, G, S, D = 8, 8, 4, a.context, 128

    # ---- inputs: R independent copies resident in HBM
    wls = [workloads.c2_decode_attention(seed=s, B=B, Hkv=Hkv, G=G, S=S, D=D) for s in range(a.copies)]
    dws = [tio.DeviceWorkload(w) for w in wls]
    virt = [pipelines.DecodeAttention(dw, materialized=False, n_splits=a.n_splits, want_lse=False) for dw in dws]
    # host cost of composing the chain into descriptors (not part of a step: maps are built once, Sec. 4.1)
    t0 = time.perf_counter()
    for _ in range(20):
        for n in ("Q", "K", "V"):
            dws[0].build(n)
    build_us = (time.perf_counter() - t0) / 20 * 1e6
    torch.cuda.synchronize()

    def mk(p):
        return lambda stream: p.run(stream)

    # the library's own choice of split count for this shape
    n_splits = a.n_splits if a.n_splits > 0 else 512 // (B * Hkv)
    alg = algorithmic_bytes_c2(B, Hkv, G, S, D, n_splits)
    wall_ms, ev_mean = time_steps(torch, [mk(p) for p in virt], a.steps, a.warmup, not a.no_graph)
    value = alg / (wall_ms * 1e-3) / 1e9
    achieved = alg / (ev_mean * 1e-3) / 1e9

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "k_decode_attn_c2_hbm_traffic.txt")
    if os.path.exists(tpath) and S == 4096:
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(float(line.split(":")[1]))
    out = {
        "metric": "virtual vs materialized latency (µs) and achieved HBM GB/s % of peak per chain",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "descriptor_build_host_us": round(build_us, 1),
        "config": {"workload": "c2: Llama-3-8B decode segment, fused QKV [8,1,6144] + KV cache [8,8,4096,128] -> "
                               "GQA 4:1 flash-decode, context 4096, Q/K/V read through descriptors",
                   "batch": B, "context": S, "kv_heads": Hkv, "q_heads": Hkv * G, "head_dim": D,
                   "input_copies_rotated": a.copies, "launch": "eager" if a.no_graph else "hip graph replay"},
        "virtual_us": round(wall_ms * 1e3, 2),
        "hbm_pct_of_peak": round(100.0 * value / HBM_PEAK_GBS, 1),
        "algorithmic_bytes": alg,
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "kernel": "k_decode_attn", "event_us_per_launch": round(ev_mean * 1e3, 2)},
    }

    if not a.no_materialized:
        mat = pipelines.DecodeAttention(dws[0], materialized=True, want_lse=False)
        torch.cuda.synchronize()
        m_steps = max(5, min(50, a.steps // 8))
        m_wall, m_ev = time_steps(torch, [mk(mat)], m_steps, 3, False)
        out["materialized_us"] = {"full": round(m_wall * 1e3, 1)}
        out["speedup_vs_materialized_full"] = round(m_wall / wall_ms, 2)
        out["intermediate_bytes_saved"] = mat.mat.bytes_written
        del mat
        torch.cuda.empty_cache()

    if a.extra:
        del virt, dws
        torch.cuda.empty_cache()
        out["chains"] = {}
        for name in a.extra.split(","):
            out["chains"][name] = chain_stats(torch, name, a_no_graph=a.no_graph, steps={"c1": 200, "c3": 30, "c4": 100, "c5": 6, "qkv_store": 200, "decode_segment": 120, "paged": 200, "moe_combine": 40}[name])
            torch.cuda.empty_cache()

    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_c2(wls[0], alg)
    print(json.dumps(out, ensure_ascii=False))


if __name__ == "__main__":
    main()
