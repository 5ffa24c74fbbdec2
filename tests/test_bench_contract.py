"""The benchmark's command-line contract: one JSON line with the agreed keys; one GPU only."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, timeout=300):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
@pytest.mark.parametrize("workload", ["C1", "V1", "T1", "E1"])
def test_one_json_line_with_roofline_and_cpu_baseline(workload):
    r = run_bench("--workload", workload, "--steps", "5", "--warmup", "2")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["vs_baseline"] is None
    assert d["higher_is_better"] is True and d["data"] == "synthetic" and d["value"] > 0 and d["ms_per_step"] > 0
    assert d["config"]["workload"].startswith(workload) and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] in ("hbm", "mfma") and rf["unit"] in ("GB/s", "TFLOP/s") and (rf["peak"] == 8000.0 or abs(rf["peak"] - 2516.6) < 0.1)
    assert rf["frac"] == pytest.approx(rf["achieved"] / rf["peak"]) and 0 < rf["frac"] < 1 and "traffic" in rf
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] == 1 and cb["value"] > 0 and cb["sample"]


@pytest.mark.gpu
def test_default_run_is_the_largest_workload_with_all_five_listed():
    r = run_bench("--steps", "20", "--warmup", "5", "--no-cpu", timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["config"]["workload"].startswith("C3") and d["roofline"]["bound"] == "mfma" and d["unit"] == "TFLOP/s"
    assert d["roofline"]["target_frac"] == 0.6 and d["roofline"]["met"] in (True, False)
    pc = d["per_config"]
    assert [c["workload"][:2] for c in pc] == ["C1", "C2", "C3", "C4", "C5"]
    for c in pc:
        assert c["avg_launch_us"] > 0 and c["tflops"] > 0 and 0 < c["frac"] < 1 and c["tuned_vs_naive"] >= 1.05
        assert c["bound"] == ("hbm" if c["workload"].startswith("C4") else "mfma")
        assert c["variant"] != "naive_1elem_per_thread"
    assert pc[2]["variant"] == d["config"]["variant"]
    assert d["tune"]["selected"] == d["config"]["variant"] and d["tune"]["log"][0]["variant"] == "naive_1elem_per_thread"
    assert all(r["parity_ok"] == 1 for r in d["tune"]["log"] if r["status"] == 0)


@pytest.mark.gpu
def test_b_given_as_n_by_k_is_a_bench_workload():
    r = run_bench("--workload", "C1", "--b-as-nk", "--steps", "20", "--warmup", "5")
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.strip()][0])
    assert "B given as [N][K]" in d["config"]["workload"]
    assert "_bnk_" in d["config"]["variant"] or "_pretransB_" in d["config"]["variant"]
    assert all(r["parity_ok"] == 1 for r in d["tune"]["log"] if r["status"] == 0)
    assert d["cpu_baseline"]["value"] > 0
