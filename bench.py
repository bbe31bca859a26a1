#!/usr/bin/env python3
"""Benchmark of the virtual-tensor hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: the consumer
kernel reading its operands through the descriptors (virtual path).  The headline workload is
the Llama-3-8B-shaped decode segment (config 2 of the benchmark spec): fused QKV output + KV cache
-> GQA flash-decoding, bf16, batch 8, context 4096.  `value`, `ms_per_step` and `roofline`
belong to it; `chains` holds, for every benchmark chain, the latency of the virtual path and of
the two materialized comparison paths (full: every operator a copy kernel; lean: only what a
stride-aware framework copies), and the chain's own roofline figure.

Inputs are resident in HBM before any timed region.  Memory-bound chains rotate over several
independent copies of their inputs so that the 256 MB Infinity Cache cannot serve them.
Short kernels are launched from HIP graphs (a Python launch costs more than they run); a sample
is then the mean launch time inside one replay.  Every timing uses HIP events on the launch
stream; virtual and materialized paths are timed the same way.

Prints one JSON line.  `--gpus N` with N > 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16/fp16 matrix peak

ALL_CHAINS = ("c1", "c3", "c4", "c5", "rowsum_large", "qkv_store", "decode_segment", "paged", "moe_combine")
DEFAULT_CHAINS = "c1,c3,c4,c5,rowsum_large,qkv_store,moe_combine,paged,decode_segment"


def algorithmic_bytes_c2(B, Hkv, G, S, D, n_splits, esz=2):
    """Bytes the method itself must move for one decode-attention step: K and V once
    (un-expanded), the fused QKV row, the output, and the split-K partial results written once
    and read once."""
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
    ap.add_argument("--copies", type=int, default=8, help="independent input copies the headline's steps rotate over")
    ap.add_argument("--no-graph", action="store_true", help="launch every step from Python instead of replaying HIP graphs")
    ap.add_argument("--no-materialized", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--n-splits", type=int, default=0, help="context splits of the attention kernel (0 = library's choice)")
    ap.add_argument("--context", type=int, default=4096, help="context length (the benchmark's is 4096; others are for tuning)")
    ap.add_argument("--copy-rates", action="store_true",
                    help="only time the copy kernels of the materialized paths on 128 MiB (and torch's device copy) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 128 MiB -> 128 MiB copy kernel 20 times (reference point for HBM byte counters)")
    ap.add_argument("--chains", default=DEFAULT_CHAINS,
                    help="comma list of the further chains to time (any of %s; 'none' for the headline alone)" % ",".join(ALL_CHAINS))
    ap.add_argument("--only-chains", action="store_true", help="skip the headline workload (for profiling one chain)")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------
# timing
# ------------------------------------------------------------------------------------------
def capture(torch, fns):
    """One HIP graph holding the launches of fns, in order."""
    stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    with torch.cuda.stream(side):
        for fn in fns:
            fn(side)                # warm the code path on the capture stream
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for fn in fns:
            fn(side)
    torch.cuda.synchronize()
    return graph


GRAPH_CAP = 512     # launches per HIP graph in the timed region
GRAPH_MIN = 32      # launches per HIP graph of the per-chain samples


def time_steps(torch, step_fns, steps, warmup, use_graph):
    """Warm-up, then EXACTLY `steps` calls of step_fns[k % R], bracketed by synchronize and by two
    HIP events on the launch stream.  With use_graph the timed region is replayed from HIP graphs
    of up to GRAPH_CAP launches each (one graph for the default 400 steps), captured beforehand: no
    step is launched from Python and a short run does not pay one graph launch per few steps.
    Returns (wall ms per step, event ms per step)."""
    R = len(step_fns)
    stream = torch.cuda.current_stream()
    graphs = {}

    def graph_of(n):
        if n not in graphs:
            graphs[n] = capture(torch, [step_fns[k % R] for k in range(n)])
        return graphs[n]

    def chunks(n):
        return [GRAPH_CAP] * (n // GRAPH_CAP) + ([n % GRAPH_CAP] if n % GRAPH_CAP else [])

    if use_graph:
        for n in set(chunks(warmup) + chunks(steps)):
            graph_of(n)

    def run(n):
        if not use_graph:
            for k in range(n):
                step_fns[k % R](stream)
            return
        for c in chunks(n):
            graph_of(c).replay()

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


def sample_launches(torch, fns, launches, use_graph, warmup=2):
    """Microseconds per launch of fns (rotating), as a list of samples.  Graph mode: a graph holds
    every fn the same number of times and at least GRAPH_MIN launches (a replay costs several
    microseconds between its events, which 8 launches per graph showed as more than 1 us per
    launch); a sample is one replay's event time divided by its launches.  Eager mode: one event
    before every launch, a sample is the time between neighbours (for kernels much longer than a
    launch from Python)."""
    stream = torch.cuda.current_stream()
    if use_graph:
        per = len(fns) * max(1, -(-GRAPH_MIN // len(fns)))
        g = capture(torch, (fns * per)[:per])
        n = max(5, -(-launches // per))
        for _ in range(warmup):
            g.replay()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        for k in range(n):
            ev[k].record()
            g.replay()
        ev[n].record()
        torch.cuda.synchronize()
        return [ev[k].elapsed_time(ev[k + 1]) * 1e3 / per for k in range(n)]
    for k in range(warmup):
        fns[k % len(fns)](stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(launches + 1)]
    torch.cuda.synchronize()
    for k in range(launches):
        ev[k].record()
        fns[k % len(fns)](stream)
    ev[launches].record()
    torch.cuda.synchronize()
    return [ev[k].elapsed_time(ev[k + 1]) * 1e3 for k in range(launches)]


def stats(samples):
    s = sorted(samples)
    return {"median": round(s[len(s) // 2], 2), "min": round(s[0], 2), "mean": round(sum(s) / len(s), 2), "samples": len(s)}


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


# chains whose full oracle pass takes seconds on the host (config 5 and the combine take tens of
# seconds and are timed by the parity tests only)
ORACLE_TIMED = ("c1", "c3", "c4", "rowsum_large", "qkv_store")


def oracle_seconds(name):
    """Wall time and cores of one full oracle pass of a chain (every operator materialized, then
    the consumer, float64 unless the paper fixes the precision), inputs generated beforehand."""
    import psutil
    import workloads
    from oracle.run import run_workload
    wl = workloads.CONFIGS[name](seed=0)
    proc = psutil.Process()
    c0 = proc.cpu_times()
    t0 = time.perf_counter()
    run_workload(wl)
    dt = time.perf_counter() - t0
    c1 = proc.cpu_times()
    cpu = (c1.user - c0.user) + (c1.system - c0.system)
    return {"seconds": round(dt, 4), "cores": max(1, int(round(cpu / dt))), "kind": "oracle", "sample": "one full pass"}


# ------------------------------------------------------------------------------------------
# the chains besides the headline
# ------------------------------------------------------------------------------------------
# name -> (input copies the virtual path rotates over, launches to sample, HIP graph?)
CHAIN_PLAN = {
    "c1": (1, 256, True),
    "c3": (3, 30, False),
    "c4": (6, 360, True),
    "c5": (1, 6, False),
    "rowsum_large": (2, 256, True),
    "qkv_store": (6, 360, True),
    "decode_segment": (4, 256, True),
    "paged": (4, 320, True),
    "moe_combine": (1, 40, False),
}


def hbm_roofline(alg_bytes, us, kernel):
    gbs = alg_bytes / (us * 1e-6) / 1e9
    return {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
            "traffic": None, "kernel": kernel}


def mfma_roofline(flops, us, kernel):
    tf = flops / (us * 1e-6) / 1e12
    r = {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
         "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None, "kernel": kernel}
    try:
        # the same against compute units x reported clock x 4096 flop per cycle (16-bit operands, dense)
        import torch
        pr = torch.cuda.get_device_properties(0)
        peak = pr.multi_processor_count * pr.clock_rate * 1e3 * 4096 / 1e12
        r["peak_at_reported_clock"] = round(peak, 1)
        r["frac_at_reported_clock"] = round(tf / peak, 4)
    except Exception:
        pass
    return r


def chain_stats(torch, name, no_graph=False, with_materialized=True):
    """Virtual, materialized-full and materialized-lean latency of one chain, and its roofline."""
    import workloads
    from paper_2604_09558_amd import pipelines
    from paper_2604_09558_amd import torch_io as tio
    copies, launches, graph_ok = CHAIN_PLAN[name]
    graph_ok = graph_ok and not no_graph
    mk = lambda p: (lambda stream: p.run(stream))      # noqa: E731
    out = {}
    lean = None
    if name == "decode_segment":
        # projection with a producer-side store + attention on the caches it wrote (Sec. 3.1)
        virt = [pipelines.DecodeSegment(*workloads.decode_segment(seed=s)) for s in range(copies)]
        M, N, K = virt[0].store.shape
        B, Hq, S, D = virt[0].attn.k.shape
        alg = (K * N + M * K + M * N) * 2 + 2 * B * (Hq // 4) * S * D * 2 + 2 * B * Hq * D * 2
        roof = lambda us: hbm_roofline(alg, us, "k_gemm_store + k_decode_attn")      # noqa: E731
        make_full = lambda i: pipelines.DecodeSegment(*workloads.decode_segment(seed=i), materialized=True)      # noqa: E731
        saved = lambda m: int(m.attn.mat.bytes_written + M * N * 2)      # noqa: E731
    else:
        maker = {"paged": workloads.paged_decode_attention, "moe_combine": workloads.moe_combine}.get(name) or workloads.CONFIGS[name]
        dws = [tio.DeviceWorkload(maker(seed=s)) for s in range(copies)]
        kw = {"want_lse": False} if name == "paged" else {}
        virt = [pipelines.make_pipeline(dw, **kw) for dw in dws]
        p0 = virt[0]
        make_full = lambda i: pipelines.make_pipeline(dws[i], materialized=True, **kw)      # noqa: E731
        saved = lambda m: int(M * N * 2) if name == "qkv_store" else int(m.mat.bytes_written)      # noqa: E731
        if name != "qkv_store":
            lean = lambda i: pipelines.make_lean_pipeline(dws[i], **kw)      # noqa: E731
        if name == "c1":
            roof = lambda us: {"bound": "launch", "note": "1.6 KB of data: latency of one launch, no roofline claim"}      # noqa: E731
        elif name in ("c3", "c5", "c4"):
            rows, N, K = sum(p0.rows), p0.N, p0.A[0].shape[-1]
            flops = 2.0 * rows * N * K
            a_bytes = rows * K * 2 if name != "c5" else dws[0].tensors["tokens"].numel() * 2
            alg = a_bytes + len(p0.B) * K * N * 2 + rows * N * 2
            if name == "c4":
                roof = lambda us: hbm_roofline(alg, us, "k_ln_gemm")      # noqa: E731
            else:
                roof = lambda us: dict(mfma_roofline(flops, us, "k_gemm"), algorithmic_bytes=int(alg))      # noqa: E731
        elif name == "rowsum_large":
            R, C = p0.x.shape
            alg = 2 * R * C * 4 + R * 4
            roof = lambda us: hbm_roofline(alg, us, "k_add_rowsum_blocks")      # noqa: E731
        elif name == "qkv_store":
            M, N, K = p0.shape
            alg = (K * N + M * K + M * N) * 2      # the weight once; rows, outputs and partial sums are small
            roof = lambda us: hbm_roofline(alg, us, "k_gemm_store")      # noqa: E731
        elif name == "moe_combine":
            R, C = p0.x.shape
            alg = 3 * R * C * 2 + R * 16
            roof = lambda us: hbm_roofline(alg, us, "k_weighted_sum_rows")      # noqa: E731
        else:   # paged
            B, Hq, S, D = p0.k.shape
            alg = 2 * B * (Hq // 4) * S * D * 2 + 2 * B * Hq * D * 2
            roof = lambda us: hbm_roofline(alg, us, "k_decode_attn")      # noqa: E731
    torch.cuda.synchronize()
    v = stats(sample_launches(torch, [mk(p) for p in virt], launches, graph_ok))
    out["virtual_us"] = v
    out["roofline"] = roof(v["median"])
    if "algorithmic_bytes" not in out["roofline"] and out["roofline"]["bound"] == "hbm":
        out["roofline"]["algorithmic_bytes"] = int(alg)
    if name in CHAIN_TRAFFIC_SOURCE:
        out["roofline"]["traffic"] = counter_traffic("chains_hbm_traffic.txt", CHAIN_TRAFFIC_SOURCE[name], key=name)
    if name == "c4":
        u = stats(sample_launches(torch, [mk(pipelines.Gemm(dw, fused=False)) for dw in dws], launches // 2, graph_ok))
        out["virtual_unfused_us"] = u
    if not with_materialized:
        return out
    # the comparison paths rotate over the same input copies (at most 3: their intermediates take memory)
    n_rot = 1 if name == "decode_segment" else min(copies, 3)
    del virt[:]
    torch.cuda.empty_cache()
    m_launches = max(3, min(launches, 24) if name != "c5" else 3)
    full = [make_full(i) for i in range(n_rot)]
    torch.cuda.synchronize()
    f = stats(sample_launches(torch, [mk(p) for p in full], m_launches, graph_ok, warmup=n_rot))
    out["materialized_full_us"] = f
    out["speedup_vs_materialized_full"] = round(f["median"] / v["median"], 3)
    out["intermediate_bytes_saved_vs_full"] = saved(full[0])
    del full
    torch.cuda.empty_cache()
    if lean is not None:
        lp = [lean(i) for i in range(n_rot)]
        torch.cuda.synchronize()
        ls = stats(sample_launches(torch, [mk(p) for p in lp], m_launches, graph_ok, warmup=n_rot))
        out["materialized_lean_us"] = ls
        out["speedup_vs_materialized_lean"] = round(ls["median"] / v["median"], 3)
        out["intermediate_bytes_saved_vs_lean"] = int(lp[0].bytes_written)
        del lp
    return out


def counter_traffic(profile_name, source_name, key=None):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None when the summary
    was made for another version of the kernel's source (it records the source's SHA-256).  A
    summary that covers several kernels labels its lines: `traffic_bytes_per_launch[key]: N`."""
    tpath = os.path.join(ROOT, "profiles", profile_name)
    spath = os.path.join(ROOT, "paper_2604_09558_amd", "csrc", source_name)
    if not (os.path.exists(tpath) and os.path.exists(spath)):
        return None
    digest = hashlib.sha256(open(spath, "rb").read()).hexdigest()
    tag = "" if key is None else "[%s]" % key
    traffic, same = None, False
    for line in open(tpath):
        if line.startswith("traffic_bytes_per_launch%s:" % tag):
            traffic = int(float(line.split(":")[1]))
        if line.startswith("source_sha256%s:" % tag):
            same = line.split(":")[1].strip() == digest
    return traffic if same else None


# chain -> source file of its dominant kernel, for the chains whose HBM counters are committed
CHAIN_TRAFFIC_SOURCE = {"c4": "vt_ln_gemm.hip", "qkv_store": "vt_gemm_store.hip", "moe_combine": "vt_kernels.hip",
                        "rowsum_large": "vt_kernels.hip", "c3": "vt_gemm.hip", "c5": "vt_gemm.hip", "paged": "vt_attn.hip"}


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
        print(json.dumps({"calibration": "vt_materialize copies 134217728 B -> 134217728 B", "launches": 20}))
        return
    if a.copy_rates:
        # the copy kernels of the materialized paths on 128 MiB, beside the runtime's device copy
        n = 128 << 20
        srcs = [torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda:0") for _ in range(4)]
        dsts = [torch.empty(n, dtype=torch.uint8, device="cuda:0") for _ in range(4)]

        def rate(fn, reps=40):
            for i in range(8):
                fn(i)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(reps):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / reps * 1e3
            return {"us": round(us, 1), "TB/s": round(2 * n / us / 1e6, 2)}

        out = {}
        flat = [vt.build_chain([], {"S": ((n // 4,), "f32", t.data_ptr())}, "S") for t in srcs]
        out["contiguous map (k_copy_flat)"] = rate(lambda i: vt.vt_materialize(flat[i % 4], dsts[i % 4]))
        out["torch copy_"] = rate(lambda i: dsts[i % 4].copy_(srcs[i % 4]))
        for name, shape in (("permute in 256-byte blocks", (4096, 128, 64)), ("permute in 1 KB blocks", (1024, 128, 256))):
            ds = [vt.build_chain([("P", "permute", ("S",), {"perm": (1, 0, 2)})], {"S": (shape, "f32", t.data_ptr())}, "P") for t in srcs]
            out[name] = rate(lambda i: vt.vt_materialize(ds[i % 4], dsts[i % 4]))
        tr = [vt.build_chain([("P", "permute", ("S",), {"perm": (1, 0)})], {"S": ((4096, 8192), "f32", t.data_ptr())}, "P") for t in srcs]
        out["transpose [4096, 8192] fp32 (k_copy_transpose)"] = rate(lambda i: vt.vt_materialize(tr[i % 4], dsts[i % 4]), reps=10)
        views = [t.view(torch.float32).view(4096, 8192).t() for t in srcs]
        outs = [t.view(torch.float32).view(8192, 4096) for t in dsts]
        out["torch copy_ of the transposed view"] = rate(lambda i: outs[i % 4].copy_(views[i % 4]), reps=10)
        print(json.dumps({"copy_rates_128MiB": out}))
        return
    chains = [] if a.chains in ("", "none") else a.chains.split(",")
    for c in chains:
        if c not in ALL_CHAINS:
            print("bench.py: unknown chain %r" % c, file=sys.stderr)
            sys.exit(2)
    B, Hkv, G, S, D = 8, 8, 4, a.context, 128

    def mk(p):
        return lambda stream: p.run(stream)

    out = {
        "metric": "virtual vs materialized latency (µs) and achieved HBM GB/s % of peak per chain",
        "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        # the paper's own end-to-end figures (abstract, Sec. 7), on other hardware and whole models: context, not a target
        "paper_context": "VTC on NVIDIA A100/H100, whole models: up to 1.93x (1.28x average) faster inference, up to 60% less memory",
    }
    wls = None
    if not a.only_chains:
        # ---- headline: config 2, R independent input copies resident in HBM
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
        n_splits = vt.vt_decode_attn_plan(virt[0].q, virt[0].k, virt[0].v, a.n_splits)["splits"]
        alg = algorithmic_bytes_c2(B, Hkv, G, S, D, n_splits)
        wall_ms, ev_ms = time_steps(torch, [mk(p) for p in virt], a.steps, a.warmup, not a.no_graph)
        per_replay = stats(sample_launches(torch, [mk(p) for p in virt], 400, not a.no_graph))
        # the same kernel on ONE input copy, which the 256 MB Infinity Cache then serves: reported
        # beside the rotating-copies figure, never used for `value` or the roofline
        warm = stats(sample_launches(torch, [mk(virt[0])], 400, not a.no_graph))
        value = alg / (wall_ms * 1e-3) / 1e9
        achieved = alg / (ev_ms * 1e-3) / 1e9
        out.update({
            "value": round(value, 1),
            "ms_per_step": round(wall_ms, 5),
            "descriptor_build_host_us": round(build_us, 1),
            "config": {"workload": "c2: Llama-3-8B decode segment, fused QKV [8,1,6144] + KV cache [8,8,4096,128] -> "
                                   "GQA 4:1 flash-decode, context 4096, Q/K/V read through descriptors",
                       "batch": B, "context": S, "kv_heads": Hkv, "q_heads": Hkv * G, "head_dim": D, "n_splits": n_splits,
                       "input_copies_rotated": a.copies, "launch": "eager" if a.no_graph else "hip graph replay"},
            "virtual_us": round(wall_ms * 1e3, 2),
            "virtual_us_per_replay": per_replay,
            "virtual_us_one_copy_cached": warm,
            "hbm_pct_of_peak": round(100.0 * value / HBM_PEAK_GBS, 1),
            "algorithmic_bytes": alg,
            "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(achieved / HBM_PEAK_GBS, 4),
                         "traffic": counter_traffic("k_decode_attn_c2_hbm_traffic.txt", "vt_attn.hip") if S == 4096 and a.n_splits == 0 else None,
                         "kernel": "k_decode_attn", "event_us_per_launch": round(ev_ms * 1e3, 2)},
        })
        if not a.no_materialized:
            del virt[1:], dws[1:]
            torch.cuda.empty_cache()
            full = pipelines.DecodeAttention(dws[0], materialized=True, want_lse=False)
            torch.cuda.synchronize()
            f = stats(sample_launches(torch, [mk(full)], 12, False, warmup=1))
            saved_full = full.mat.bytes_written
            del full
            torch.cuda.empty_cache()
            lean = pipelines.make_lean_pipeline(tio.DeviceWorkload(wls[0]), want_lse=False)
            torch.cuda.synchronize()
            ls = stats(sample_launches(torch, [mk(lean)], 12, False, warmup=1))
            out["materialized_us"] = {"full": f["median"], "lean": ls["median"], "full_min": f["min"], "lean_min": ls["min"]}
            out["speedup_vs_materialized_full"] = round(f["median"] / (ev_ms * 1e3), 2)
            out["speedup_vs_materialized_lean"] = round(ls["median"] / (ev_ms * 1e3), 2)
            out["intermediate_bytes_saved"] = saved_full
            out["intermediate_bytes_saved_vs_lean"] = int(lean.bytes_written)
            del lean
        del virt, dws
        torch.cuda.empty_cache()

    if chains:
        out["chains"] = {}
        for name in chains:
            t0 = time.perf_counter()
            try:
                out["chains"][name] = chain_stats(torch, name, no_graph=a.no_graph, with_materialized=not a.no_materialized)
            except Exception as e:      # one chain must not take the whole line down; the failure is reported in its place
                out["chains"][name] = {"error": "%s: %s" % (type(e).__name__, e)}
            out["chains"][name]["bench_seconds"] = round(time.perf_counter() - t0, 1)
            torch.cuda.empty_cache()
            if not a.no_cpu_baseline and name in ORACLE_TIMED:
                try:
                    out["chains"][name]["cpu_baseline"] = oracle_seconds(name)
                except Exception as e:
                    out["chains"][name]["cpu_baseline"] = {"error": "%s: %s" % (type(e).__name__, e)}

    if not a.no_cpu_baseline and wls is not None:
        out["cpu_baseline"] = cpu_baseline_c2(wls[0], alg)
    print(json.dumps(out, ensure_ascii=False))


if __name__ == "__main__":
    main()
