"""Host logic of bench.py that needs no GPU: the one-GPU rule, the loud failure without a GPU (no CPU fallback),
and the planner leg, which is host only."""
import json
import subprocess
import sys
from pathlib import Path

import pytest
import torch

ROOT = Path(__file__).resolve().parent.parent


def bench(*args):
    return subprocess.run([sys.executable, str(ROOT / "bench.py"), *args], cwd=ROOT, capture_output=True, text=True,
                          timeout=300)


@pytest.mark.parametrize("n", ["2", "8"])
def test_more_than_one_gpu_is_refused_with_a_message(n):
    r = bench("--gpus", n)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the behaviour of a machine without a GPU")
@pytest.mark.parametrize("args", [(), ("--kv-commit",), ("--config", "3"), ("--paper-sampling", "qwen3")])
def test_without_a_gpu_the_compute_legs_fail_loudly(args):
    r = bench(*args)
    assert r.returncode == 2
    assert "no GPU visible" in r.stderr and r.stdout.strip() == ""       # no number from any CPU path


def test_planner_leg_prints_one_json_line():
    r = bench("--planner")
    assert r.returncode == 0, r.stderr
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "cpu_baseline"):
        assert key in out
    assert out["value"] > 0 and out["cpu_baseline"]["kind"] == "oracle" and "workload" in out["config"]


def test_unknown_sampling_setting_is_refused():
    r = bench("--paper-sampling", "llama")
    assert r.returncode == 2 and "invalid choice" in r.stderr and r.stdout.strip() == ""
