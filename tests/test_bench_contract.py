"""bench.py's command line and the one JSON line it prints."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


@pytest.mark.gpu
@pytest.mark.parametrize("extra", [[], ["--rope"], ["--block"]])
def test_json_line_has_the_agreed_fields(extra):
    r = subprocess.run([sys.executable, BENCH, "--config", "0", "--steps", "3", "--warmup", "1"] + extra,
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 3 and j["warmup"] == 1 and j["vs_baseline"] is None
    assert j["data"] == "synthetic" and "workload" in j["config"] and j["value"] > 0
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in j["roofline"], key
    assert abs(j["roofline"]["frac"] - j["roofline"]["achieved"] / j["roofline"]["peak"]) < 1e-3
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in j["cpu_baseline"], key
    assert j["cpu_baseline"]["kind"] == "oracle"
    assert j["cpu_baseline"]["gpu_max_rel_err_vs_oracle_seq0"] <= 1e-4       # config 0 is the fp32 case
