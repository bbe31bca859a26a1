"""Per-workgroup timelines of the hand-scheduled kernels on the benchmark's workloads.

Needs the profiling build of the library (`python -m paper_2604_09558_amd.build --profile`, which
compiles the same sources with -DVT_PROFILE into libvt_profile.so): its kernels mark a few points
per workgroup with the 100 MHz wall clock, and this script prints when those points are reached
(min / median / max over the workgroups, microseconds from the first workgroup's start) and how
the compute dies compare.  The marks cost a little time: read the ordinary library's duration
from rocprofv3, and the shape of the timeline from here.

    python -m paper_2604_09558_amd.profile_trace attn [--n-splits N] [--reps R]
    python -m paper_2604_09558_amd.profile_trace gemm | gemm_store | ln_gemm | add_rowsum | layernorm
    python -m paper_2604_09558_amd.profile_trace gemm_values     (k_gemm's duration and clock against the operand values)
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

from paper_2604_09558_amd import binding  # noqa: E402

assert binding._lib is None, "the library is already loaded"
binding.LIB_PATH = os.path.join(HERE, "libvt_profile.so")       # every call below goes to the profiling build

SLOTS = 8
MARKS = {
    "attn": ["start", "first K tile staged", "tile loop done", "partial results stored", "ticket taken",
             "merge written", "merge loads landed"],
    "gemm": ["start", "first tiles in LDS", "K loop done", "tile stored"],
    "gemm_store": ["start", "first tile multiplied", "tile loop done", "partial sums stored", "ticket taken", "mapped store done"],
    "add_rowsum": ["start", "maps in LDS", "block addresses known", "first 512 columns added", "row written"],
    "layernorm": ["start", "map in LDS", "row addresses known", "first rows loaded", "first rows stored", "all stores complete"],
    "ln_gemm": ["start", "first two blocks requested", "W in registers", "first block multiplied", "last block multiplied",
                "last stores issued", "all memory operations complete"],
}


def read_marks(lib, kernel, n_wg):
    buf = (C.c_longlong * (n_wg * SLOTS))()
    fn = getattr(lib, "vt_profile_read_" + kernel)
    fn.argtypes = [C.POINTER(C.c_longlong), C.c_int]
    rc = fn(buf, n_wg)
    if rc != 0:
        raise RuntimeError("vt_profile_read_%s failed (%d)" % (kernel, rc))
    rate = getattr(lib, "vt_profile_ticks_per_us_" + kernel)
    rate.restype = C.c_double
    return np.array(buf[:], dtype=np.int64).reshape(n_wg, SLOTS), float(rate())


def report(kernel, marks):
    t, ticks_per_us = marks
    xcc = t[:, 7]
    t0 = t[:, 0][t[:, 0] > 0].min()
    fresh = (t[:, :7] > 0) & (t[:, :7] >= t[:, 0:1])       # marks older than the workgroup's own start are a previous launch's
    us = np.where(fresh, (t[:, :7] - t0) / ticks_per_us, np.nan)
    for k, name in enumerate(MARKS[kernel]):
        col = us[:, k][~np.isnan(us[:, k])]
        if col.size:
            print("  %-24s min %6.2f  median %6.2f  max %6.2f   (%d workgroups)" % (name, col.min(), np.median(col), col.max(), col.size))
    if kernel == "attn":
        m = ~np.isnan(us[:, 5])                       # the workgroups that merged
        steps = [("tile loop done -> partial results stored", 2, 3), ("-> ticket taken", 3, 4), ("-> merge loads landed", 4, 6),
                 ("-> merge written", 6, 5)]
        print("  merging workgroups, median step: " + "; ".join("%s %.2f" % (n, np.median(us[m, b] - us[m, a])) for n, a, b in steps))
        print("  last mark of the launch %.2f us = last tile loop done %.2f + %.2f" % (
            np.nanmax(us[:, 5]), np.nanmax(us[:, 2]), np.nanmax(us[:, 5]) - np.nanmax(us[:, 2])))
    k_done = {"add_rowsum": 4, "layernorm": 5}.get(kernel, 2)
    print("  '%s' by compute die (median / max): " % MARKS[kernel][k_done] +
          "  ".join("%d: %.1f/%.1f" % (x, np.nanmedian(us[xcc == x, k_done]), np.nanmax(us[xcc == x, k_done]))
                    for x in sorted(set(xcc.tolist()))))
    print("  workgroups per compute die: " + " ".join("%d:%d" % (x, int((xcc == x).sum())) for x in sorted(set(xcc.tolist()))))


def trace_attn(a):
    import torch
    import workloads
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io as tio
    lib = vt.lib()
    copies = [tio.DeviceWorkload(workloads.c2_decode_attention(seed=s)) for s in range(4)]
    ps = [pipelines.DecodeAttention(dw, n_splits=a.n_splits, want_lse=False) for dw in copies]
    plan = vt.vt_decode_attn_plan(ps[0].q, ps[0].k, ps[0].v, a.n_splits)
    B, Hq, S, D = ps[0].k.shape
    n_wg = plan["splits"] * (Hq // plan["group_size"]) * B
    for _ in range(3):
        for p in ps:
            p.run()
    torch.cuda.synchronize()
    read_marks(lib, "attn", n_wg)
    for rep in range(a.reps):
        # three launches on other input copies push this one's K/V out of the caches; the marks kept are the last launch's
        for p in (ps[2], ps[3], ps[0]):
            p.run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ps[1].run()
        e1.record()
        torch.cuda.synchronize()
        print("config 2, %d workgroups (%d splits), launch %d: %.1f us between events" % (n_wg, plan["splits"], rep, e0.elapsed_time(e1) * 1e3))
        report("attn", read_marks(lib, "attn", n_wg))


def trace_gemm(a):
    """Config 3 (o-proj GEMM 8192 x 4096 x 4096): phases of every 256 x 256 tile."""
    import torch
    import workloads
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io as tio
    lib = vt.lib()
    ps = [pipelines.Gemm(tio.DeviceWorkload(workloads.c3_oproj_gemm(seed=s))) for s in range(2)]
    n_wg = 512
    for p in ps:
        p.run()
    torch.cuda.synchronize()
    read_marks(lib, "gemm", n_wg)
    for rep in range(a.reps):
        ps[1].run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ps[0].run()
        e1.record()
        torch.cuda.synchronize()
        print("config 3, %d workgroups, launch %d: %.1f us between events" % (n_wg, rep, e0.elapsed_time(e1) * 1e3))
        t, rate = read_marks(lib, "gemm", n_wg)
        report("gemm", (t, rate))
        us = (t[:, :4] - t[:, 0:1]) / rate
        print("  per tile, median (max): load-in %.1f (%.1f), K loop %.1f (%.1f), store %.1f (%.1f) us" % (
            np.median(us[:, 1]), us[:, 1].max(), np.median(us[:, 2] - us[:, 1]), (us[:, 2] - us[:, 1]).max(),
            np.median(us[:, 3] - us[:, 2]), (us[:, 3] - us[:, 2]).max()))
        ghz = (t[:, 5] - t[:, 4]) / ((t[:, 2] - t[:, 1]) / rate) / 1e3
        print("  shader cycle counter over the K loop: %.3f GHz median (%.3f .. %.3f)" % (np.median(ghz), ghz.min(), ghz.max()))


def trace_ln_gemm(a):
    """Config 4 (window partition -> LayerNorm -> linear 128 -> 384, fp16): the persistent workgroups' phases."""
    import torch
    import workloads
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io as tio
    lib = vt.lib()
    ps = [pipelines.make_pipeline(tio.DeviceWorkload(workloads.c4_window_ln_linear(seed=s))) for s in range(4)]
    n_wg = 256
    for p in ps:
        p.run()
    torch.cuda.synchronize()
    read_marks(lib, "ln_gemm", n_wg)
    for rep in range(a.reps):
        for p in (ps[2], ps[3], ps[0]):
            p.run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ps[1].run()
        e1.record()
        torch.cuda.synchronize()
        print("config 4, %d workgroups, launch %d: %.1f us between events" % (n_wg, rep, e0.elapsed_time(e1) * 1e3))
        t, rate = read_marks(lib, "ln_gemm", n_wg)
        report("ln_gemm", (t, rate))
        us = (t[:, :7] - t[:, 0:1].min()) / rate
        seven = us[:, 4] > np.median(us[:, 4]) + 1.0
        print("  workgroups with one more block: %d; their 'last block multiplied' median %.2f, the others' %.2f" % (
            int(seven.sum()), np.median(us[seven, 4]) if seven.any() else float("nan"), np.median(us[~seven, 4])))


def trace_gemm_values(a):
    """Config 3's shape with dense operands of different VALUES: the matrix cores draw less power
    on zeros than on random data, and the clock the chip grants follows.  Prints, per kind of data,
    the duration of 20 back-to-back launches (three times), the shader clock over the K loop of the
    last launch, and the duration of torch.matmul (the vendor library) on the same operands."""
    import torch
    import paper_2604_09558_amd as vt
    lib = vt.lib()
    M, K, N, n_wg = 8192, 4096, 4096, 512
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    zeros = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    normal = lambda *s: torch.randn(*s, generator=gen, device="cuda").to(torch.bfloat16)
    c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")

    def timed(fn):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        out = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                fn()
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / 20 * 1e3)
        return out

    print("8192 x 4096 x 4096, bf16, dense operands; us per launch over 20 launches (three runs), marks included")
    for name, a_, b_ in (("zeros", zeros(M, K), zeros(K, N)), ("ones", zeros(M, K) + 1, zeros(K, N) + 1),
                         ("A normal, B zeros", normal(M, K), zeros(K, N)), ("normal", normal(M, K), normal(K, N))):
        A = vt.build_chain([], {"A": ((M, K), "bf16", a_.data_ptr())}, "A")
        B = vt.build_chain([], {"B": ((K, N), "bf16", b_.data_ptr())}, "B")
        ts = timed(lambda: vt.vt_gemm([A], [B], [c], "bf16"))
        t, rate = read_marks(lib, "gemm", n_wg)
        ghz = (t[:, 5] - t[:, 4]) / ((t[:, 2] - t[:, 1]) / rate) / 1e3
        ref = timed(lambda: torch.matmul(a_, b_, out=c))
        flops = 2.0 * M * N * K
        print("  %-18s k_gemm %s us (best %.0f TFLOP/s), K-loop clock %.3f GHz median | torch.matmul %s us (best %.0f TFLOP/s)" % (
            name, " ".join("%.1f" % x for x in ts), flops / min(ts) / 1e6, np.median(ghz),
            " ".join("%.1f" % x for x in ref), flops / min(ref) / 1e6), flush=True)


def trace_gemm_store(a):
    """The decode-step QKV projection [8,4096] x [4096,6144] with the producer-side store."""
    import torch
    import workloads
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io as tio
    lib = vt.lib()
    ps = [pipelines.GemmStore(tio.DeviceWorkload(workloads.qkv_proj_store(seed=s))) for s in range(4)]
    n_wg = 4096
    for p in ps:
        p.run()
    torch.cuda.synchronize()
    read_marks(lib, "gemm_store", n_wg)
    for rep in range(a.reps):
        for p in (ps[2], ps[3], ps[0]):
            p.run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ps[1].run()
        e1.record()
        torch.cuda.synchronize()
        t, rate = read_marks(lib, "gemm_store", n_wg)
        live = t[:, 0] > 0
        print("qkv projection store, %d workgroups, launch %d: %.1f us between events" % (int(live.sum()), rep, e0.elapsed_time(e1) * 1e3))
        report("gemm_store", (t[live], rate))


def trace_add_rowsum(a):
    """The add + row-sum consumer on the 335 MB chain (first wave of each workgroup of four rows)."""
    import torch
    import workloads
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import pipelines, torch_io as tio
    lib = vt.lib()
    ps = [pipelines.make_pipeline(tio.DeviceWorkload(workloads.rowsum_chain_large(seed=s))) for s in range(3)]
    n_wg = 2048
    for p in ps:
        p.run()
    torch.cuda.synchronize()
    read_marks(lib, "add_rowsum", n_wg)
    for rep in range(a.reps):
        for p in (ps[2], ps[0]):
            p.run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ps[1].run()
        e1.record()
        torch.cuda.synchronize()
        t, rate = read_marks(lib, "add_rowsum", n_wg)
        live = t[:, 0] > 0
        print("add + row-sum, %d workgroups, launch %d: %.1f us between events" % (int(live.sum()), rep, e0.elapsed_time(e1) * 1e3))
        report("add_rowsum", (t[live], rate))


def trace_layernorm(a):
    """The LayerNorm consumer on config 4's window-partitioned rows (first wave of each workgroup of 128 rows)."""
    import torch
    import workloads
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import torch_io as tio
    lib = vt.lib()
    dws = [tio.DeviceWorkload(workloads.c4_window_ln_linear(seed=s)) for s in range(3)]
    ds = [d.build("T") for d in dws]
    outs = [d.empty(ds[0].shape) for d in dws]
    n_wg = 1024
    for i in range(3):
        vt.vt_elementwise(vt.EW_LAYERNORM, ds[i], None, 1e-5, outs[i])
    torch.cuda.synchronize()
    read_marks(lib, "layernorm", n_wg)
    for rep in range(a.reps):
        for i in (2, 0):
            vt.vt_elementwise(vt.EW_LAYERNORM, ds[i], None, 1e-5, outs[i])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        vt.vt_elementwise(vt.EW_LAYERNORM, ds[1], None, 1e-5, outs[1])
        e1.record()
        torch.cuda.synchronize()
        t, rate = read_marks(lib, "layernorm", n_wg)
        live = t[:, 0] > 0
        print("layernorm, %d workgroups, launch %d: %.1f us between events" % (int(live.sum()), rep, e0.elapsed_time(e1) * 1e3))
        report("layernorm", (t[live], rate))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("kernel", choices=sorted(MARKS) + ["gemm_values"])
    ap.add_argument("--n-splits", type=int, default=0)
    ap.add_argument("--reps", type=int, default=3)
    a = ap.parse_args()
    {"attn": trace_attn, "gemm": trace_gemm, "gemm_store": trace_gemm_store, "gemm_values": trace_gemm_values,
     "ln_gemm": trace_ln_gemm, "add_rowsum": trace_add_rowsum, "layernorm": trace_layernorm}[a.kernel](a)


if __name__ == "__main__":
    main()
