"""bench.py's contract: one GPU only (a larger --gpus is refused with a message), and on a GPU the
one JSON line carries the metric, the roofline and the oracle baseline objects and the extra step
shapes. The GPU case runs the small `tiny` workload so that it takes seconds."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, timeout=600):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, stdout=subprocess.PIPE,
                          stderr=subprocess.PIPE, text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused():
    res = _run("--gpus", "2")
    assert res.returncode == 2 and "one GPU" in res.stderr and not res.stdout.strip()


@pytest.mark.gpu
def test_json_line_on_the_tiny_workload():
    print("case bench.py --workload tiny", flush=True)
    res = _run("--workload", "tiny", "--steps", "3", "--warmup", "1", "--cpu-sample-layers", "1")
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "step_alg1_us",
                "step_gather_free_us", "seeds", "breakdown_us_per_step"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["unit"] == "us/step" and d["higher_is_better"] is False
    assert d["vs_baseline"] is None and "workload" in d["config"] and d["config"]["workload"].startswith("tiny")
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and r["stream_read_ceiling_gbps"] > 1000
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
    assert abs(d["value"] - d["ms_per_step"] * 1e3) < 1.0


@pytest.mark.gpu
def test_draft_budget_sweep_mode():
    print("case bench.py --draft-budgets", flush=True)
    res = _run("--workload", "tiny", "--draft-budgets", "256,512")
    assert res.returncode == 0, res.stderr[-2000:]
    d = json.loads([l for l in res.stdout.splitlines() if l.startswith("{")][0])
    assert [e["budget"] for e in d["sweep"]] == [256, 512]
    assert all(e["us_per_call_mean"] > 0 and e["kv_len"] == e["budget"] + 3 for e in d["sweep"])
