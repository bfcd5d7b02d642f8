"""Host-side checks of the benchmark's command line contract (no GPU needed)."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_unknown_workload_is_refused():
    r = run_bench("--workload", "9")
    assert r.returncode != 0 and "invalid choice" in r.stderr


def test_traffic_summary_is_valid_json_with_the_fields_bench_reads():
    with open(os.path.join(ROOT, "profiles", "spmm_rmat1m_d128_f32_hbm_traffic.json")) as f:
        d = json.load(f)
    assert d["hbm_bytes_per_spmm_call"] > 1e9
    assert abs(d["calibration"]["fetch_scale"] - 2.0) < 0.05 and abs(d["calibration"]["write_scale"] - 1.0) < 0.05
