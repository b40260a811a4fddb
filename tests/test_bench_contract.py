"""bench.py's command-line contract: one GPU only; one JSON line with the agreed fields."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_json_line_on_the_small_config():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "c1", "--steps", "5", "--warmup", "1"],
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "configs", "achievable", "kernels",
                "schedule_report"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 1 and d["data"] == "synthetic"
    assert d["vs_baseline"] is None and d["higher_is_better"] is True and "workload" in d["config"]
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert abs(roof["frac_cold"] - roof["achieved_cold"] / roof["peak"]) < 1e-3
    assert roof["launches_timed"] >= 20 and "median_launch_ms" in roof and "recorded" in roof["traffic_source"]
    assert d["config"]["instrumented_allreduces"] >= 20
    # one record per other configuration, each with the steady-state and the flushed-cache figures
    assert [c["id"] for c in d["configs"]] == ["c2-lane", "c2-ring", "c3", "c4"]
    for c in d["configs"]:
        for key in ("workload", "ms_per_allreduce", "GBps", "frac_of_peak", "ms_per_allreduce_cold", "frac_cold",
                    "dominant_kernel", "kernels", "launches_timed_per_kernel"):
            assert key in c, (c["id"], key)
        assert c["launches_timed_per_kernel"] >= 20
        assert 0 < c["frac_cold"] < 1 and 0 < c["dominant_kernel"]["frac_cold"] < 1
        assert abs(c["frac_of_peak"] - c["GBps"] / 8000.0) < 1e-3
    ach = d["achievable"]
    for key in ("stream_copy_GBps", "add_2_operands_in_place_GBps", "reduce_8_operands_in_place_GBps",
                "dominant_kernel_over_best_ceiling"):
        assert ach[key] > 0, key
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    one = cpu["single_thread"]
    assert one["cores"] == 1 and one["value"] > 0 and one["seconds"] > 0


def test_default_workload_is_the_largest_fp32_configuration():
    """The timed line is taken on config 5 (1024 ranks, 4 GiB resident), the configuration whose
    rates are DRAM rates; the traffic figure it quotes comes from the committed counter summary."""
    sys.path.insert(0, ROOT)
    import bench

    saved = sys.argv
    try:
        sys.argv = ["bench.py"]
        args = bench.parse()
    finally:
        sys.argv = saved
    assert args.config == "c5" and args.gpus == 1 and args.steps >= 20 and args.warmup >= 3
    cfg = bench.CONFIGS["c5"]
    assert cfg["topo"] == (32, 4, 8) and cfg["n"] == 1 << 20 and cfg["dtype"] == "float32" and cfg["algo"] == "lane_multiproc"
    assert bench.INSTRUMENTED >= 20
    t = bench.recorded_traffic("c5", "lane_multiproc", "S1")
    assert t is not None and 0.99 < t / ((1024 + 32) * (1 << 20) * 4) < 1.02  # (P + N) n e algorithmic bytes
    assert bench.recorded_traffic("c5", "lane_multiproc", "no such stage") is None
