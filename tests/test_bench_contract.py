"""bench.py's host-side contract, without a GPU: argument handling, the statistics helpers, the
record skeleton, and the refusal of more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU only" in r.stderr and r.stdout.strip() == ""


def test_defaults_are_one_gpu_and_a_short_run(monkeypatch):
    monkeypatch.setattr(sys, "argv", ["bench.py"])
    a = bench.parse()
    assert a.gpus == 1 and 1 <= a.steps <= 50 and 0 <= a.warmup <= 10 and a.workload == bench.HEADLINE
    assert not a.no_other_workloads and not a.no_ceiling and not a.k_sweep


def test_stats_are_mean_median_min():
    s = bench._stats([4.0, 1.0, 2.0, 9.0])
    assert s == {"avg_ms": 4.0, "median_ms": 3.0, "min_ms": 1.0}
    assert bench._stats([5.0, 7.0, 6.0])["median_ms"] == 6.0
    e = bench._kernel_entry([2.0, 2.0], 58, 1_000_000)
    assert e["bytes_per_param"] == 58 and e["GBps"] == pytest.approx(58e6 / 2e-3 / 1e9)
    assert e["frac"] == pytest.approx(e["GBps"] / bench.HBM_PEAK_GBS) and e["GBps_best"] == e["GBps_median"] == e["GBps"]


def test_record_skeleton_has_the_contract_keys():
    from paper_2512_17570_amd import inputs as I

    class Props:
        name, multi_processor_count, total_memory = "x", 256, 1

    wl = I.WORKLOADS[bench.HEADLINE]
    rec = bench._base_record(wl, Props, 1.0, 20, 5, 2.0, {"tensor_sets": 1})
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config"):
        assert key in rec
    assert rec["n_gpus"] == 1 and rec["vs_baseline"] is None and rec["dtype"] == "f32" and rec["data"] == "synthetic"
    assert rec["config"]["workload"] == bench.HEADLINE and "model" not in rec["config"]
    assert rec["config"]["n_params"] == 805_412_864 and rec["config"]["k_grad_buffers"] == 16
    json.dumps(rec)


def test_stored_traffic_figure_is_the_one_in_the_profile():
    """roofline.traffic is a stored rocprofv3 figure: it has to be the one the profile summary derives."""
    text = open(os.path.join(ROOT, "profiles", "gs_step_gpt65b_layer_h8192_k16.txt")).read()
    want = f"{bench.MEASURED_TRAFFIC_BYTES[bench.HEADLINE]:,}".replace(",", " ")
    assert want in text
    assert abs(bench.MEASURED_TRAFFIC_BYTES[bench.HEADLINE] / (58 * 805_412_864) - 1.0) < 1e-3
