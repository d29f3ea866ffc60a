"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figures_name_their_profile_and_sources():
    sys.path.insert(0, ROOT)
    import bench
    assert len(bench.kernel_sources_sha16()) == 16
    for name, rec in bench.MEASURED_TRAFFIC.items():
        assert rec["bytes"] > 0 and len(rec["csrc_sha16"]) == 16
        assert os.path.isfile(os.path.join(ROOT, rec["profile"])), rec["profile"]
        # the profile file quotes the same source hash the figure is tied to
        assert rec["csrc_sha16"] in open(os.path.join(ROOT, rec["profile"])).read(), (name, rec["profile"])
    # a figure is only reported for the sources it was measured on
    got, src = bench.measured_traffic("no_such_workload")
    assert got is None
