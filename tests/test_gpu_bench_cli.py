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


def test_default_line_carries_the_call_forms_and_the_other_workloads():
    """The command the benchmark is run with (fewer steps): the headline workload's record, the same step through the
    three named calls and as two parties, and short runs of workloads 1, 3, 4 and 5 with their own parity checks."""
    d = run_bench("--steps", "40", "--warmup", "8", "--cpu-seconds", "0.2")
    assert d["config"]["workload"].startswith("config2") and d["config"]["mode"] == "fused" and d["parity"]["ok"]
    src = d["roofline"]["traffic_source"]      # None if the stored summary is of another kernel instance
    assert (src is None) == (d["roofline"]["traffic"] is None) and (src is None or src["file"].startswith("profiles/"))
    for key in ("three_calls", "two_parties"):
        assert d[key]["us_per_step"] > 0 and d[key]["GBps"] > 0
    others = d["other_workloads"]
    assert [o["workload"].split(":")[0] for o in others] == ["config1", "config3", "config4", "config5"]
    for o in others:
        assert o["us_per_step"] > 0 and 0 < o["roofline_frac"] < 1 and o["parity"]["ok"], o
    # the sub-records are the default workload's only
    assert "other_workloads" not in run_bench(*SMALL)
