"""Host logic of bench.py that needs no GPU: the refusal of more than one GPU, and the tie between the measured
HBM traffic it prints and the kernel sources that figure was measured with."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
    assert not r.stdout.strip().startswith("{")          # no JSON line that could be taken for a measurement


def test_measured_traffic_belongs_to_the_sources_and_the_workload():
    sys.path.insert(0, ROOT)
    import bench
    m = bench.MEASURED_TRAFFIC
    # the figure is printed only for the launch and the kernel sources it was measured with ...
    assert bench.measured_traffic(m["bytes_per_step"] + 50) is None
    # ... and the sources in the tree are those: a change to the Slice-and-Scale kernel or the device header without a
    # new counter profile fails here instead of leaving `roofline.traffic` null in the next run
    assert bench.kernel_sources_hash() == m["sources_sha256"], "mx_ss.hip / mx_device.h changed: re-measure FETCH_SIZE / WRITE_SIZE (profiles/) and update MEASURED_TRAFFIC"
    assert bench.measured_traffic(m["bytes_per_step"]) == m["bytes"]
    assert 1.0 <= m["bytes"] / m["bytes_per_step"] < 1.01  # HBM traffic within 1 % of the algorithmic bytes
