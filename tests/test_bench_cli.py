"""bench.py's command line: what can be checked without a GPU, and the JSON line on one."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, timeout=600):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    out = _run("--gpus", "2")
    assert out.returncode == 2 and "ONE GPU" in out.stderr and out.stdout == ""


def test_without_a_gpu_it_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    out = _run("--workload", "c0")
    assert out.returncode == 1 and "no GPU" in out.stderr and out.stdout == ""


@pytest.mark.gpu
def test_json_line_on_the_small_workload():
    """One JSON line with the fields the contract names, the roofline object and the CPU baseline."""
    out = _run("--workload", "c0", "--steps", "3", "--warmup", "1", "--cpu-sample", str(1 << 20), "--no-cpu-full-configs",
               "--graph")
    assert out.returncode == 0, out.stderr
    lines = [l for l in out.stdout.split("\n") if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["unit"] == "params/s" and d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["higher_is_better"] is True
    assert d["config"]["workload"].startswith("c0") and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and r["achieved"] > 0
    assert abs(d["value"] - d["config"]["params"] / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "params/s" and c["cores"] >= 1 and c["value"] > 0
    assert r["traffic"] is None and r["traffic_source"] is None          # no counter reading is carried for c0
    e = d["end_to_end_with_gradient_generation"]
    assert e["ms_per_step"] >= 0.5 * d["ms_per_step"] and e["steps"] >= 1
    g = d["hip_graph"]
    assert g["ms_per_step"] > 0 and g["params_per_s"] > 0


@pytest.mark.gpu
def test_two_builds_compared_in_one_process():
    """--compare-lib steps the same state with two builds of the library in turn (here: the in-tree build
    against itself) and prints the per-round times of both."""
    from paper_2309_12381_amd import build
    out = _run("--workload", "c1", "--steps", "3", "--compare-lib", build.LIB)
    assert out.returncode == 0, out.stderr
    lines = [l for l in out.stdout.split("\n") if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["unit"] == "ms" and d["steps_per_round"] == 3 and d["config"]["workload"] == "c1"
    assert len(d["ms_per_step"]["in_tree"]) == 4 and len(d["ms_per_step"]["other"]) == 4
    assert all(x > 0 for k in ("in_tree", "other") for x in d["ms_per_step"][k])
    assert 0.5 < d["other_over_in_tree"] < 2.0


@pytest.mark.gpu
def test_c_interface_alone_steps_a_small_llama_shape():
    """--c-caller: a program that uses only include/mpo.h and include/mpo_probe.h (no Python, no PyTorch in its
    process) allocates, places, plans and steps a Llama-shaped list and reports a plausible rate."""
    out = _run("--c-caller", "--shape", "2048", "5504", "6", "32000", "--steps", "5")
    assert out.returncode == 0, out.stderr
    d = json.loads(out.stdout.strip())
    params = 2 * 32000 * 2048 + 6 * (2 * 2048 + 4 * 2048 * 2048 + 3 * 2048 * 5504) + 2048
    assert d["params"] == params and d["tensors"] == 1 + 9 * 6 + 2 and d["launches_per_step"] == 9 and d["steps"] == 5
    assert 2000.0 < d["GBps"] < 8000.0 and abs(d["frac_of_peak"] - d["GBps"] / 8000.0) < 1e-3
    assert d["placement"]["searched"] is True and d["placement"]["candidates"] >= 1
