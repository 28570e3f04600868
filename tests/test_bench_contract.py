"""bench.py prints one JSON line with the agreed fields (run on a small workload so that it takes seconds)."""
import json
import os
import subprocess
import sys

import pytest

from conftest import ROOT, say

pytestmark = pytest.mark.gpu


def run_bench(*args):
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), *args]
    say("running " + " ".join(cmd[1:]))
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=280)
    return res


def test_bench_line_has_the_agreed_fields():
    res = run_bench("--workload", "gpt125m", "--steps", "3", "--warmup", "1", "--cpu-budget", "1")
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [ln for ln in res.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["unit"] == "params/s" and d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1
    assert d["vs_baseline"] is None and d["higher_is_better"] is True and d["data"] == "synthetic"
    assert d["config"]["workload"] == "gpt125m" and "model" not in d["config"]
    assert abs(d["value"] - d["config"]["params"] / (d["ms_per_step"] * 1e-3)) <= 1e-6 * d["value"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and 0 < r["frac"] < 1
    # the default path is the speculative just-in-time one; bytes are what was moved, the algorithmic figure beside it
    assert d["config"]["path"] == "spec" and d["config"]["algorithmic_bytes_per_param_step"] == 19
    assert 17.0 <= d["config"]["bytes_per_param_step"] <= 20.0 and d["speculation"]["steps"] == 3
    assert "jit" in d["other_paths"] and d["other_paths"]["jit"]["bytes_per_param_step"] == 19
    # memory-only skeletons of the four kernels, timed on the same buffers
    for name in ("amax", "cast", "adam_amax", "adam_update", "update_reads_only", "update_writes_only"):
        assert d["ceilings"][name]["GBps"] > 0
    assert 0 < d["kernels"]["adam_update"]["frac_of_skeleton"] <= 1.1
    assert d["config"]["placement"]["allocation"]            # where the buffers were put, and how that was decided
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "params/s" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
    assert d["value"] > 100 * c["value"]                     # the GPU path, not the oracle, was timed as `value`


def test_bench_refuses_more_than_one_gpu():
    res = run_bench("--gpus", "2")
    assert res.returncode != 0 and "one GPU" in res.stderr
