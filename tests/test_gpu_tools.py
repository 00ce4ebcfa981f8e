"""The measuring scripts at the repository root share code (sweep.py uses bench.py's layers,
graph capture and timers): one small run of each path that a change to either could break."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.gpu


def test_sweep_measures_a_small_shape():
    import torch
    sys.path.insert(0, ROOT)
    import sweep
    from paper_2509_12211_amd import tinyserve as ts, workloads as wl
    spec = wl.scaled(wl.SPECS["tiny"], L=2048, topk=16)
    r = sweep.measure(torch, ts, wl, spec, 16, "cuda:0")
    assert r["step_us"] > 0 and r["dense_us"] > 0
    assert 0.0 < r["mass_captured_mean"] <= 1.0 + 1e-6
    assert r["K"] == 16 and r["S"] == spec.S


def test_bench_prints_one_json_line_for_a_single_workload():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "tiny", "--steps", "32",
                          "--warmup", "8", "--no-cpu-baseline", "--no-all-workloads", "--no-extras"],
                         capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert out.returncode == 0, out.stderr[-2000:]
    lines = [l for l in out.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["n_gpus"] == 1 and d["value"] > 0 and d["roofline"]["frac"] > 0
    assert d["steps"] >= 32 and d["config"]["workload"].startswith("configs[")
