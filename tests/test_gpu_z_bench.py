"""The benchmark's contract on a GPU machine: one JSON line with the agreed fields (short runs)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*extra):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "8", "--warmup", "2",
                        "--no-cpu-baseline", *extra], capture_output=True, text=True, timeout=280)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    return json.loads(lines[0])


def _check_common(d):
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 8 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and "workload" in d["config"]
    assert abs(d["value"] - d["config"]["total_query_tokens"] / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12 and 0.05 < rf["frac"] < 1.0
    assert rf["traffic"] is None or rf["traffic"] >= 0.9 * rf["algorithmic_bytes"]


def test_bench_line_hot_path():
    d = _run("--hot-path-only")
    _check_common(d)
    assert d["config"]["workload"] == "cfg3-llama3-8b-gqa" and d["dtype"] == "bf16"
    assert d["config"]["accept_kernel_path"] == "two_pass"
    assert d["roofline_accept"]["algorithmic_bytes"] < d["roofline_accept"]["per_row_form_bytes"]


def test_bench_line_tree():
    d = _run("--tree", "3")
    _check_common(d)
    assert d["config"]["workload"].endswith("-tree3") and d["config"]["tree"]["max_children_per_node"] == 3
    assert "walk" in d["config"]["accept_kernel_path"]


def test_bench_line_default_has_every_config():
    """The default line (what the driver records): the headline workload, the benchmark's other
    configurations and the policy-shaped batch, each with its step time and fractions."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "12", "--warmup", "3"],
                       capture_output=True, text=True, timeout=580)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    assert d["config"]["workload"] == "cfg3-llama3-8b-gqa" and d["steps"] == 12
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["value"] > 0 and d["cpu_baseline"]["cores"] >= 1
    assert d["accept_vs_oracle"]["hard_mismatches"] == 0
    assert set(d["other_configs"]) == {"cfg2", "cfg4", "cfg4g", "cfg5"}
    for name, o in d["other_configs"].items():
        assert o["ms_per_step"] > 0 and 0.02 < o["attention_frac"] < 1.0 and 0.0 < o["accept_frac"] < 1.0, (name, o)
        assert o["accept_vs_oracle"]["hard_mismatches"] == 0, (name, o)
    p = d["policy_preset"]
    assert p["workload"].endswith("-policy") and p["draft_steps"] >= 1 and p["accept_vs_oracle"]["hard_mismatches"] == 0
    assert sum(p["spec_len_histogram"]) == p["batch"]
