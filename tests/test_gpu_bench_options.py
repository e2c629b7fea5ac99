"""bench.py's measurement options on a truncated stack (4 layers of the headline shard): the JSON line's contract,
the chained step's timeline and the pipeline-stage run.  The figures are not the metric (4 of 80 layers)."""
import json
import os
import subprocess
import sys

import pytest
import torch

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*flags):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--mode", "decode", "--layers", "4", "--steps", "8", "--warmup", "2",
           "--reps", "1", "--no-cpu", "--no-ceiling", *flags]
    print("[bench options]", " ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [ln for ln in res.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1, res.stdout[-2000:]
    return json.loads(lines[0])


def test_decode_line_and_timeline():
    r = run_bench("--timeline")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
                "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 8 and r["config"]["workload"] == "70b_r8_decode" and r["value"] > 0
    assert r["roofline"]["bound"] == "hbm" and 0 < r["roofline"]["frac"] < 1 and r["roofline"]["launches"] == 8   # one launch per step
    t = r["timeline"]
    assert t["unit"] == "us" and t["blocks_recorded"] > 0 and t["period_per_layer"] > 0
    assert set(t["first_ready_to_last_end"]) == {"attention", "qkv", "o", "gate_up", "down"}
    assert t["phase_attention_o_beside_gate_up"] > 0 and t["phase_qkv_beside_down"] > 0


def test_pipeline_stage_run():
    one = run_bench("--stages", "1")
    two = run_bench("--stages", "2")
    assert one["config"]["pipeline_stages"] == 1 and two["config"]["layers_per_stage"] == [2, 2]
    assert 0 < one["ms_per_step"] < two["ms_per_step"] * 1.5 and two["value"] > 0
