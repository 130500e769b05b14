"""bench.py's command-line contract: one GPU only, no CPU fallback, one JSON line with the agreed fields."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def _run(*args, timeout=600):
    return subprocess.run([sys.executable, BENCH, *args], capture_output=True, text=True, timeout=timeout, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_no_gpu_means_no_result():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode == 2 and "no CPU fallback" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_json_line_fields_on_the_small_layer():
    r = _run("--workload", "tiny_fp32", "--steps", "3", "--warmup", "1", "--cpu-sample-tokens", "64")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 3 and j["warmup"] == 1 and j["unit"] == "tokens/s"
    assert j["warmup_steps_run"] >= j["warmup"]          # warm-up goes on until the clocks have settled
    assert j["config"]["workload"] == "tiny_fp32" and j["dtype"] == "f32" and j["data"] == "synthetic"
    assert abs(j["value"] - j["config"]["T"] / (j["ms_per_step"] * 1e-3)) <= 1e-3 * j["value"]
    rf = j["roofline"]
    assert rf["bound"] in ("hbm", "mfma", "alu") and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert j["ceilings"]["stream_read_GB/s"] > 0 and j["ceilings"]["stream_read_bytes"] > 0
    assert len(rf["launch_ms_p10_p50_p90"]) == 3 and set(j["layer"]["calls_rates"]) == set(j["layer"]["calls_ms"])
    assert sum(j["config"]["tokens_per_expert"]) == j["config"]["T"] * j["config"]["k"]
    cpu = j["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0


@pytest.mark.gpu
def test_default_run_carries_the_whole_curve():
    """No --workload: the headline workload plus the Mixtral-shaped sweep (both roofline regimes) and the
    micro-batch study, still as ONE JSON line that honours --steps and --warmup."""
    r = _run("--steps", "2", "--warmup", "1", "--cpu-sample-tokens", "16")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    assert j["config"]["workload"] == "mixtral_T256" and j["steps"] == 2 and j["warmup"] == 1
    assert [e["T"] for e in j["sweep"]] == [32, 64, 128, 256, 512, 1024, 2048, 4096]
    for e in j["sweep"]:
        f = e["ffn_input"]
        assert f["bound"] in ("hbm", "mfma") and abs(f["frac"] - f["achieved"] / f["peak"]) < 1e-3
        assert abs(e["tokens_per_s"] - e["T"] / (e["ms_per_step"] * 1e-3)) <= 1e-3 * e["tokens_per_s"]
    at256 = next(e for e in j["sweep"] if e["T"] == 256)
    assert at256["ms_per_step"] == j["ms_per_step"] and at256["ffn_input"]["frac"] == j["roofline"]["frac"]
    assert j["sweep"][0]["ffn_input"]["bound"] == "hbm" and j["sweep"][-1]["ffn_input"]["bound"] == "mfma"
    big = j["roofline_large_batch"]
    assert big["workload"] == "mixtral_T4096" and big["bound"] == "mfma" and big["unit"] == "TFLOP/s"
    assert j["roofline"]["traffic"] is None or "profiles/" in j["roofline"]["traffic_source"]
    mb = j["micro_batch_study"]
    assert mb["workload"] == "finegrained_T8192" and [row["m"] for row in mb["rows"]] == [1, 2, 3, 4]
    assert all(row["two_stream_ms_per_step"] > 0 for row in mb["rows"])
    assert j["cpu_baseline"]["gflops"] > 0 and j["cpu_baseline"]["cores_source"]


@pytest.mark.gpu
def test_router_gate_times_the_layer_from_the_gating_gemm():
    r = _run("--workload", "tiny_fp32", "--router", "gate", "--steps", "3", "--warmup", "1", "--cpu-sample-tokens", "64")
    assert r.returncode == 0, r.stderr[-2000:]
    j = json.loads([l for l in r.stdout.splitlines() if l.strip()][-1])
    assert "gating GEMM" in j["config"]["router"]
    assert {"gate_route", "gate_route_dispatch", "ffn_input", "ffn_output", "combine"} == set(j["layer"]["calls_ms"])
    assert sum(j["config"]["tokens_per_expert"]) == j["config"]["T"] * j["config"]["k"]
