"""bench.py's contract with its driver: one JSON line with the agreed keys; one GPU only."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KEYS = {"metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
        "dtype", "data", "config", "roofline", "cpu_baseline"}


def _run(*args, timeout=600):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True, text=True,
                          timeout=timeout)


def _last_json(stdout):
    lines = [l for l in stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, "bench.py prints exactly one JSON line"
    return json.loads(lines[0])


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2", timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_prefix_cache_workload_runs_on_the_host_and_keeps_the_keys():
    r = _run("--workload", "prefix-cache")
    assert r.returncode == 0, r.stderr[-2000:]
    d = _last_json(r.stdout)
    assert KEYS <= set(d), sorted(KEYS - set(d))
    assert d["n_gpus"] == 0 and d["vs_baseline"] is None   # the manager is host code: no GPU is used
    assert "workload" in d["config"] and "model" not in d["config"]
    assert d["value"] > 1.0                      # shared keys keep fewer blocks resident than per-adapter keys
    assert d["cpu_baseline"]["kind"] == "oracle"


@pytest.mark.gpu
def test_small_decode_workload_prints_roofline_and_cpu_baseline():
    r = _run("--workload", "c3-small", "--steps", "3", "--warmup", "1")
    assert r.returncode == 0, r.stderr[-2000:]
    d = _last_json(r.stdout)
    assert KEYS <= set(d), sorted(KEYS - set(d))
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["unit"] == "tokens/s" and d["value"] > 0 and d["ms_per_step"] > 0
    rf = d["roofline"]
    assert {"bound", "achieved", "peak", "unit", "frac", "traffic"} <= set(rf)
    assert rf["bound"] in ("hbm", "mfma", "alu") and rf["peak"] > 0
    if rf["achieved"] is not None:   # at the reduced size a launch-bound row kernel may dominate: no roofline for it
        assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-6
    cb = d["cpu_baseline"]
    assert {"value", "unit", "cores", "kind", "sample"} <= set(cb) and cb["kind"] == "oracle" and cb["cores"] >= 1
