"""bench.py's command line on the GPU: every mode runs on a small workload and prints the one JSON line with the keys
the benchmark contract names."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SMALL = ["--config", "2", "--users", "3", "--lens", "40,700,0,300", "--steps", "16", "--warmup", "8", "--cpu-seconds", "0.05"]


def run_bench(*args):
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-3000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, res.stdout[-2000:]          # exactly one line on stdout
    return json.loads(lines[0])


@pytest.mark.parametrize("extra", [
    [],
    ["--mode", "calls"],
    ["--mode", "two_parties"],
    ["--mode", "streams"],
    ["--append", "--lens", "40,700,1,300"],
    ["--graph", "--copies", "4"],
    ["--decode-loop", "8"],
    ["--mode", "per_user_streams", "--graph", "--copies", "2"],
    ["--mode", "two_processes", "--user-procs", "2"],
    ["--mode", "two_processes", "--user-procs", "1"],
], ids=lambda e: "_".join(x.strip("-") for x in e) or "fused")
def test_bench_modes_on_a_small_workload(extra):
    d = run_bench(*SMALL, *extra)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 16 and d["value"] > 0 and d["config"]["workload"].startswith("config2")
    assert set(d["roofline"]) >= {"bound", "achieved", "peak", "unit", "frac", "traffic"}
    if "--decode-loop" not in extra:
        assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["cores"] >= 1
        assert d["parity"]["ok"], d["parity"]


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT,
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert res.returncode != 0 and "one GPU" in res.stderr
