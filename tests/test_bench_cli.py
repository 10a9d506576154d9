"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line that could be taken for a measurement


def test_help_needs_no_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "--steps" in r.stdout and "--warmup" in r.stdout


def test_traffic_figures_come_from_a_committed_profile_summary():
    """roofline.traffic is whatever the rocprofv3 summary under profiles/ says, or null: no
    constant in bench.py."""
    sys.path.insert(0, ROOT)
    import bench
    traffic, src = bench.read_traffic("cfg2")
    assert src == os.path.join("profiles", "pmc_cfg2.md")
    assert os.path.exists(os.path.join(ROOT, src))
    # within a percent of the algorithmic bytes of the cfg2 passes (n p 4 and n p 4 + 4 n)
    assert abs(traffic["fa_gram_kernel"] / 6.72e8 - 1) < 0.01
    assert abs(traffic["fa_combine_kernel"] / 7.168e8 - 1) < 0.01
    assert bench.read_traffic("no_such_workload") == ({}, None)
    assert bench.read_traffic(None) == ({}, None)
    assert "MEASURED_TRAFFIC" not in open(os.path.join(ROOT, "bench.py")).read()
