"""Host-side checks of bench.py's contract that need no GPU."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figure_comes_from_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    txt = open(bench.TRAFFIC_FILE).read()
    # the summary states the commands that produced it and the kernel source it was measured on
    assert "rocprofv3 --pmc FETCH_SIZE" in txt and "rocprofv3 --pmc WRITE_SIZE" in txt
    stamp = [l.split(":")[1].strip() for l in txt.splitlines() if l.startswith("kernel_source_sha256_16:")]
    assert len(stamp) == 1 and len(stamp[0]) == 16
    t = bench.read_traffic(source_hash=stamp[0])
    assert t is not None and 128 * 2 ** 20 <= t <= 4 * 128 * 2 ** 20      # at least the algorithmic bytes of a launch
    # a figure measured on another version of the kernel is not reported
    assert bench.read_traffic(source_hash="0" * 16) is None
    assert bench.read_traffic() in (None, t)


def test_workload_named_by_bench_is_the_metric_configuration():
    sys.path.insert(0, ROOT)
    import bench
    base = json.load(open(os.path.join(ROOT, "BASELINE.json")))
    from workloads import workload
    w = workload(bench.WORKLOAD)
    assert (w.B, w.Hq, w.Hkv, w.N, w.d, w.causal) == (1, 28, 4, 8192, 128, True)
    assert "N=8192" in base["configs"][2] and "Hq=28" in base["configs"][2]       # the configuration the metric's target is quoted on
