"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode == 2
    assert "one GPU" in p.stderr
    assert p.stdout.strip() == ""              # no JSON line for a run that did not happen


def test_traffic_figure_comes_from_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.measured_traffic("cfg3")
    # the update reads the fp32 matrix and writes it and a bf16 copy: 262 MB at the very least
    assert t is not None and 2.6e8 < t < 6e8
    text = open(os.path.join(ROOT, "profiles", "cfg3_update_kernel_hbm_traffic.txt")).read()
    assert "rocprofv3 --pmc FETCH_SIZE" in text and "rocprofv3 --pmc WRITE_SIZE" in text
    assert bench.measured_traffic("no-such-workload") is None
