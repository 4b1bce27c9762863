"""Host-side checks of bench.py's contract that need no GPU."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_default_workload_is_the_largest_layer():
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert 'ap.add_argument("--workload", default="c5"' in src
    B = _bench_module()
    assert {"c2", "c3", "c4", "c5"} <= set(B.WORKLOADS)
    assert "57344" in B.WORKLOADS["c5"] and "16384" in B.WORKLOADS["c4"]


def test_traffic_is_reported_only_for_the_build_it_was_read_on():
    B = _bench_module()
    versions = {k[2] for k in B.MEASURED_TRAFFIC_KIB}
    assert len(versions) == 1                         # every reading belongs to one library version
    v = versions.pop()
    assert B.traffic_for("c5", "tiled", v) == sum(B.MEASURED_TRAFFIC_KIB[("c5", "tiled", v)]) * 1024
    assert B.traffic_for("c5", "tiled", v + ".1") is None
    assert B.traffic_for("c5", "canonical", v) is None
    assert B.traffic_for("c3", "tiled", v) is None


def test_peaks_are_the_published_ones():
    B = _bench_module()
    assert (B.PEAK_FP4_TFLOPS, B.PEAK_F16_TFLOPS, B.PEAK_HBM_GBS) == (10100.0, 2500.0, 8000.0)
