"""The benchmark's one-line JSON contract, on a short run (no 128K pass, no extras, no CPU oracle)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_prints_one_json_line_with_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "64", "--warmup", "16",
                        "--no-long", "--no-extras", "--no-cpu"], capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 64 and d["warmup"] == 16
    assert d["higher_is_better"] is False and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    assert abs(d["ms_per_step"] * 1e3 - d["value"]) < 1e-2
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert 0.05 < rf["frac"] < 1.0 and 1.0 < d["value"] < 1000.0
    # the ceiling measured in the same process, the label's single source of truth, and the traffic's provenance
    assert 4000.0 < rf["measured_peak"] < 8000.0 and abs(rf["frac_of_measured"] - rf["achieved"] / rf["measured_peak"]) < 1e-3
    assert rf["kernel"].startswith("fb::attn_stream_kernel<128, 0, 0, 4>")
    assert rf["traffic"] is None or "not measured in this run" in rf["traffic_source"]
    assert rf["launches_timed"] >= 30 and rf["min_launch_us"] <= rf["median_launch_us"]
    cal = d["calibration"]
    assert cal["mfma_bf16_TFLOPs"] < cal["mfma_bf16_TFLOPs_constant_operands"] <= 2600.0
    assert d["timing"]["repeats"] >= 5
    # parity of this very run against the oracle, inside the stated tolerances by a wide margin
    par = d["parity"]
    assert par["tiny_f32"]["max_abs_err_out"] < 1e-5 and par["tiny_f32"]["max_abs_err_L_ext"] < 1e-5
    assert par["llm_32k"]["max_abs_err_out"] < 1e-3 and par["llm_32k"]["max_abs_err_L_ext"] < 1e-3


def test_gamma_calibration_report():
    """Head-wise selective reuse on synthetic drift: similarity falls with the drift rate, the threshold splits
    the heads, refreshed heads match full recomputation, reused heads stay far closer to it than the refreshed
    heads would if they were reused too, and refreshing a subset of heads is faster than refreshing all."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gamma-calibration"],
                       capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([ln for ln in r.stdout.splitlines() if ln.strip()][-1])
    sim = d["mean_similarity_by_head"]
    assert all(a >= b - 1e-3 for a, b in zip(sim, sim[1:])) and sim[0] > 0.99 and sim[-1] < 0.85
    assert 0 < d["refreshed_heads_per_reuse_step"] < len(sim)
    assert d["l1_to_full_recompute_refreshed_heads"] < 1e-3
    assert d["l1_to_full_recompute_reuse_heads"] < 0.2 * d["l1_of_those_heads_if_they_were_reused_too"]
    assert d["external_us_selected_heads"] < 0.6 * d["external_us_all_heads"]


def test_tau_policy_report():
    """The updated-token-count rule on a synthetic unmasking schedule: a larger threshold refreshes less often,
    costs less attention time per step and drifts further from full recomputation."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--tau-policy"],
                       capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([ln for ln in r.stdout.splitlines() if ln.strip()][-1])
    rows = d["by_tau"]
    assert [x["tau"] for x in rows[:3]] == [1, 2, 3] and rows[-1]["refresh_fraction"] == 1.0
    fr = [x["refresh_fraction"] for x in rows[:4]]
    us = [x["attention_us_per_step"] for x in rows[:4]]
    l1 = [x["l1_to_full_recompute"] for x in rows[:4]]
    assert fr == sorted(fr, reverse=True) and abs(fr[3] - 0.125) < 1e-9
    assert us == sorted(us, reverse=True) and us[0] < rows[-1]["attention_us_per_step"]
    assert l1 == sorted(l1) and l1[3] < 0.05 * d["mean_abs_output"]
