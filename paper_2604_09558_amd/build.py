"""Compile the HIP sources of this package into libvt.so (in-tree, gfx950)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libvt.so")
LIB_PROFILE = os.path.join(HERE, "libvt_profile.so")   # same sources with -DVT_PROFILE: per-workgroup timestamps

HOST_SOURCES = ["vt_build.cpp", "vt_device_host.cpp", "vt_vtog.cpp"]
HIP_SOURCES = ["vt_kernels.hip", "vt_attn.hip", "vt_gemm.hip", "vt_ln_gemm.hip", "vt_gemm_store.hip"]

COMMON = ["-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC, "-Wall", "-Wno-unused-function"]
# gfx950 only; packed-fp32 instructions are switched off (they have given wrong results on
# the target machines), the compiler still emits ordinary fp32 code.
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unknown-warning-option", "-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics"]
# Kernels whose waits count vector memory operations by hand, or whose speed depends on their
# register budget: a spill (scratch) would add memory operations the counts do not know of.
# The build fails if the compiler reports scratch for any of them.
NO_SCRATCH = ("k_decode_attn", "k_ln_gemm", "k_gemm_store", "k_gemm")


def scratch_report(compiler_output: str):
    """[(kernel, scratch bytes per lane)] from the compiler's kernel-resource-usage remarks."""
    res, name = [], None
    for line in compiler_output.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line and name:
            res.append((name, int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])))
            name = None
    return res


def hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(verbose: bool = True, jobs: int = 4, profile: bool = False) -> str:
    """Compile and link libvt.so, or with profile=True libvt_profile.so (the kernels record
    per-workgroup timestamps that profile_trace.py reads; load it through VT_LIB_PATH)."""
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    tag = ".prof" if profile else ""
    lib = LIB_PROFILE if profile else LIB
    for src in HOST_SOURCES + HIP_SOURCES:
        obj = os.path.join(HERE, "_build", src + tag + ".o")
        cmd = [hipcc()] + COMMON + (["-DVT_PROFILE"] if profile else []) + (DEVICE if src.endswith(".hip") else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print("[build]", " ".join(cmd), flush=True)
        # the compiler's remarks go to a file: a pipe that nobody reads while the build waits for
        # another compiler would fill up and stall this one
        log = open(obj + ".log", "w+")
        procs.append((src, subprocess.Popen(cmd, stdout=log, stderr=subprocess.STDOUT, text=True), log))
        objs.append(obj)
        while sum(p.poll() is None for _, p, _ in procs) >= jobs:
            for _, p, _ in procs:
                if p.poll() is None:
                    p.wait()
                    break
    failed = False
    for src, p, log in procs:
        p.wait()
        log.seek(0)
        out = log.read()
        log.close()
        for kernel, scratch in scratch_report(out):
            if scratch and any(k in kernel for k in NO_SCRATCH):
                print("[build] FAILED: %s uses %d bytes of scratch per lane (%s)" % (kernel, scratch, src), file=sys.stderr)
                failed = True
        out = "\n".join(l for l in out.splitlines() if "-Rpass-analysis=kernel-resource-usage" not in l
                        and "is not a recognized feature" not in l)
        if out.strip() and verbose:
            print(out)
        if p.returncode != 0:
            print("[build] FAILED:", src, file=sys.stderr)
            if not verbose:
                print(out, file=sys.stderr)
            failed = True
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib] + objs
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return lib


def build_ceilings(verbose: bool = True) -> str:
    """Compile csrc/vt_ceilings.hip, a standalone program that measures what plain kernels with the
    consumers' access patterns reach on the machine (no part of the library; nothing loads it)."""
    exe = os.path.join(HERE, "vt_ceilings")
    cmd = [hipcc(), "-O3", "-std=c++17"] + DEVICE[:5] + ["-o", exe, os.path.join(CSRC, "vt_ceilings.hip")]
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    text = "\n".join(l for l in out.stdout.splitlines() if "is not a recognized feature" not in l)
    if text.strip() and verbose:
        print(text)
    if out.returncode != 0:
        raise RuntimeError("hipcc failed on vt_ceilings.hip")
    return exe


if __name__ == "__main__":
    if "--ceilings" in sys.argv:
        build_ceilings()
    else:
        build(profile="--profile" in sys.argv)
