"""The benchmark's output line, end to end on the smallest workload: one JSON line with the contract's fields,
the roofline and CPU-baseline objects, and the in-process comparison of the push's span orders."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + list(args), capture_output=True, text=True,
                       cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, r.stdout[-2000:]
    return json.loads(lines[0])


@pytest.mark.gpu
def test_bench_line_on_the_tiny_workload():
    d = _run("--workload", "tiny", "--steps", "6", "--warmup", "2", "--ab-push-order", "list,win4,mix8,split2")
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 6 and d["warmup"] == 2 and d["config"]["workload"].startswith("tiny:")
    assert d["value"] > 0 and d["ms_per_step"] > 0 and d["ms_per_step_median"] > 0
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12
    assert rf["frac_of_copy_ceiling"] > 0 and d["copy_ceiling_GBps"] > 1000
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    ab = d["push_order_ab"]
    assert set(ab) == {"list", "win4", "mix8", "split2"}
    assert all(v["push_ms_median"] > 0 and v["step_ms_median"] > 0 for v in ab.values())
    assert set(d["stage_ms"]) == {"probe", "insert", "pool", "sort", "push", "fixup", "merge", "order"}


@pytest.mark.gpu
def test_bench_kstep_line_reports_the_merge():
    d = _run("--workload", "kstep", "--steps", "4", "--warmup", "4", "--no-cpu-baseline")
    assert d["roofline"]["kernel"] == "k_merge" and d["roofline"]["algorithmic_bytes_per_launch"] > 0
    assert d["stage_launches_per_step"]["merge"] == 0.25


@pytest.mark.gpu
@pytest.mark.parametrize("args", [
    ["--workload", "tiny", "--variant", "adagrad"],
    ["--workload", "tiny", "--variant", "kingma"],
    ["--workload", "tiny", "--grad-bf16"],
    ["--workload", "tiny", "--push-order", "split4", "--no-cpu-baseline"],
    ["--workload", "tiny", "--seam"],
    ["--workload", "kstep", "--variant", "prose", "--no-cpu-baseline"],
])
def test_bench_modes_print_one_line(args):
    d = _run(*(args + ["--steps", "4", "--warmup", "4"]))
    assert d["value"] > 0 and d["ms_per_step"] > 0 and d["n_gpus"] == 1


@pytest.mark.gpu
@pytest.mark.parametrize("args", [["--workload", "tiny", "--variant", "prose"], ["--workload", "kstep", "--variant", "adagrad"],
                                  ["--workload", "tiny", "--predict"]])
def test_bench_refuses_combinations_it_does_not_time(args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + args, capture_output=True, text=True, cwd=ROOT,
                       timeout=600)
    assert r.returncode == 2 and r.stdout.strip() == "" and "bench.py:" in r.stderr
