"""The library's host logic (descriptor builder, contiguity and block analysis, device-form
converter with the kernels' evaluator run on the CPU, opportunity graph and greedy search) built
with AddressSanitizer and UndefinedBehaviorSanitizer and run under the host tests.

Only the three host sources are compiled (g++, no GPU toolchain); the kernel entry points are
stand-ins that answer "no device" (tests/support/host_only_stubs.cpp), so the tests that need a
real kernel entry point's host checks are left out of this run.  The tests run in a child
interpreter with the sanitizer runtime preloaded; any report makes the child fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_09558_amd", "csrc")
HOST_SOURCES = ["vt_build.cpp", "vt_device_host.cpp", "vt_vtog.cpp"]
NEED_DEVICE_UNITS = ["test_error_paths", "test_store_maps_must_be_one_to_one", "test_attention_plan_of_the_decode_chain",
                     "test_attention_group_size_divides_the_broadcast_factor", "test_attention_plan_recognises_page_tables",
                     "test_attention_plan_rejects_what_the_kernel_cannot_read"]


def gcc_file(name):
    return subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True, check=True).stdout.strip()


def test_host_logic_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan, stdcxx = gcc_file("libasan.so"), gcc_file("libstdc++.so")
    if not (os.path.isabs(asan) and os.path.exists(asan)):
        pytest.skip("no sanitizer runtime in this toolchain")
    lib = str(tmp_path / "libvt_host_san.so")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
           "-fno-sanitize-recover=undefined", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-I", "/opt/rocm/include", "-w"] + [os.path.join(CSRC, f) for f in HOST_SOURCES] + [
               os.path.join(ROOT, "tests", "support", "host_only_stubs.cpp"), "-o", lib]
    subprocess.run(cmd, check=True, timeout=600)
    env = dict(os.environ, LD_PRELOAD=asan + " " + stdcxx, VT_LIB_PATH=lib, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = [sys.executable, "-m", "pytest", "-q", "-p", "no:cacheprovider", "-x",
           os.path.join(ROOT, "tests", "test_descriptor_host.py"), os.path.join(ROOT, "tests", "test_vtog.py")]
    for name in NEED_DEVICE_UNITS:
        run += ["--deselect", "tests/test_descriptor_host.py::" + name]
    r = subprocess.run(run, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, tail
    assert " passed" in r.stdout
