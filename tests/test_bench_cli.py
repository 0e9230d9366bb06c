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


import json

import pytest


@pytest.mark.gpu
def test_the_bench_line_keeps_its_contract():
    """One JSON line on stdout with the fields the driver reads, the roofline of the dominant kernel
    and the oracle's CPU baseline (short run: 30 timed steps, 2 oracle steps)."""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "30", "--warmup", "5",
                        "--cpu-steps", "2"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 30 and d["warmup"] == 5 and d["higher_is_better"] is True
    assert d["unit"] == "coded layer-steps/s" and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert abs(d["value"] * d["ms_per_step"] - 1000.0) < 1e-6 * 1000.0
    assert d["config"]["workload"].startswith("cfg3") and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and 0.05 < r["frac"] < 1.0
    assert abs(r["achieved"] - r["algorithmic_bytes"] / (r["avg_launch_ms"] * 1e-3) / 1e9) < 1e-6 * r["achieved"]
    assert r["traffic"] is None or r["traffic"] > r["algorithmic_bytes"] * 0.9
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["unit"] == d["unit"] and c["sample"]
    assert sum(d["verdicts"].values()) == 60 and d["verified_checks_agree"] is True
    assert r["avg_launch_samples"] >= 4                      # the dominant kernel is bracketed on 4 timed steps of a short run (8 of a long one)
    p = d["roofline_products"]                               # the coded GEMMs against the MFMA peak of their arithmetic
    assert p["bound"] == "mfma" and p["unit"] == "TFLOP/s" and p["peak"] == 2500.0 and p["samples"] >= 2
    assert abs(p["frac"] - p["achieved"] / p["peak"]) < 1e-9 and 0.02 < p["frac"] < 1.0
    assert abs(p["frac_forward"] - p["flops_forward"] / (p["forward_ms"] * 1e-3) / 1e12 / p["peak"]) < 1e-9


@pytest.mark.gpu
def test_the_mlp_bench_line():
    """cfg2 (784-1024-1024-10) as whole training iterations: layer-steps per second, the verdicts
    that the fault lists imply (one parity block only detects: every faulty product is reported
    UNCORRECTABLE and computed again, clean the second time), overhead against the uncoded run."""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "cfg2", "--steps", "6", "--warmup", "2",
                        "--cpu-steps", "2"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    assert d["unit"] == "coded layer-steps/s" and d["config"]["layers"] == 3 and d["steps"] == 6
    assert abs(d["value"] * d["ms_per_step"] - 1000.0) < 1e-6 * 1000.0
    assert abs(d["ms_per_iteration"] - 3 * d["ms_per_step"]) < 1e-9
    v = d["verdicts"]
    assert v["corrected"] == 0 and v["uncorrectable"] > 0
    assert v["clean"] == 6 * 6                               # every product ends clean: 3 layers x 2 products x 6 iterations
    assert d["coding_overhead"] > d["coding_overhead_without_faults"] > 0.0
    assert d["roofline"]["bound"] == "mfma" and d["cpu_baseline"]["kind"] == "oracle"


@pytest.mark.gpu
def test_the_strategy_comparison_leg():
    """CodeNet, replication and uncoded on the cfg2 network for 20 iterations each: CodeNet and
    replication end with the weights of a run without errors (to float32 accuracy / exactly), uncoded
    does not; the expected-time model is quoted both ways next to the measured times."""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--strategies", "--steps", "20", "--fault-p", "0.0015"],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    d = json.loads([l for l in p.stdout.splitlines() if l.strip()][0])
    cod, rep, unc = (d["strategies"][k] for k in ("codenet", "replication", "uncoded"))
    done = [r for r in cod["sweep"] if r["finished"]]
    assert done and all(max(r["distance_from_fault_free_run"]) < 1e-3 for r in done)
    assert any(r["classes"]["corrected"] > 0 for r in done)
    done = [r for r in rep["sweep"] if r["finished"]]
    assert done and all(max(r["distance_from_fault_free_run"]) == 0.0 for r in done)
    assert all(r["classes"]["corrected"] == 0 for r in rep["sweep"])
    assert max(unc["relative_distance_of_final_weights_from_the_fault_free_run"]) > 1e-3
    assert d["replication_over_codenet_measured"] > 1.0
    assert all("model_seconds_chain" in r and "model_seconds_as_printed" in r for r in done)
