"""bench.py's command line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_a_multi_rank_launch_is_refused_too():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0", LOCAL_RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode != 0 and "single-GPU" in r.stderr


def test_counter_traffic_is_tied_to_the_kernel_source():
    """roofline.traffic comes from a committed counter summary that records the SHA-256 of the
    kernel's source: for the committed pair the figure is reported, for any other source it is not."""
    sys.path.insert(0, ROOT)
    import bench
    t = bench.counter_traffic("k_decode_attn_c2_hbm_traffic.txt", "vt_attn.hip")
    assert t is not None and 136_511_488 <= t <= 1.02 * 136_511_488, t      # nothing read twice
    assert bench.counter_traffic("k_decode_attn_c2_hbm_traffic.txt", "vt_gemm.hip") is None     # another source: stale
    assert bench.counter_traffic("no_such_file.txt", "vt_attn.hip") is None


def test_chain_traffic_entries_are_keyed_and_tied_to_their_sources():
    """The chains' counter summary holds one labelled entry per chain; each is reported only for the
    source file whose hash it records, and none of the memory-bound ones shows re-reads (traffic
    within 6 % above the algorithmic bytes the summary states beside it)."""
    sys.path.insert(0, ROOT)
    import re
    import bench
    text = open(os.path.join(ROOT, "profiles", "chains_hbm_traffic.txt")).read()
    alg = [int(m) for m in re.findall(r"algorithmic (\d+) B", text)]
    assert len(alg) == len(bench.CHAIN_TRAFFIC_SOURCE) == 7
    for (key, src), a in zip(bench.CHAIN_TRAFFIC_SOURCE.items(), alg):
        t = bench.counter_traffic("chains_hbm_traffic.txt", src, key=key)
        if t is None:       # the kernel's source changed after the counters were read: bench reports null
            continue
        if key in ("c3", "c5"):     # the GEMM's panels are read once per compute die and round (not HBM-bound)
            assert a <= t, (key, t, a)
        else:
            assert a <= t <= 1.06 * a, (key, t, a)      # the projection's partial sums of five K slices are 5 % of its bytes
        assert bench.counter_traffic("chains_hbm_traffic.txt", "vt_build.cpp", key=key) is None      # another source: stale
    assert bench.counter_traffic("chains_hbm_traffic.txt", "vt_kernels.hip", key="no_such_chain") is None
    assert bench.counter_traffic("chains_hbm_traffic.txt", "vt_kernels.hip") is None      # unlabelled lines: none in this file
