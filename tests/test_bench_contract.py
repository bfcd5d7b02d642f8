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


def test_traffic_summaries_are_valid_json_with_the_fields_bench_reads():
    sys.path.insert(0, ROOT)
    import bench
    for name, least in (("spmm_rmat1m_d128_f32_hbm_traffic.json", 1e9), ("spmm_rmat1m_d128_bf16_hbm_traffic.json", 1e9),
                        ("spmm_clustered5a_d256_bf16_hbm_traffic.json", 1e8)):
        with open(os.path.join(ROOT, "profiles", name)) as f:
            d = json.load(f)
        assert d["hbm_bytes_per_spmm_call"] > least
        assert abs(d["calibration"]["fetch_scale"] - 2.0) < 0.05 and abs(d["calibration"]["write_scale"] - 1.0) < 0.05
        # the summary names the kernel sources it was measured with, by the same list bench.py hashes
        assert sorted(d["sources"]) == sorted(bench.TRAFFIC_SOURCES) and d["kernels"]


def test_a_counter_figure_is_dropped_when_the_kernel_sources_differ(monkeypatch):
    sys.path.insert(0, ROOT)
    import bench
    monkeypatch.setattr(bench, "source_hashes", lambda: {k: "0" * 16 for k in bench.TRAFFIC_SOURCES})
    value, why = bench.read_traffic("4", "f32")
    assert value is None and "changed" in why
    assert bench.read_traffic("2", "f32")[0] is None
