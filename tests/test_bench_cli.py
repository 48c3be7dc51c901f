"""bench.py's command line on a machine without a GPU: more than one GPU is refused with a message,
and without a GPU the benchmark stops instead of falling back to anything."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused():
    r = run("--gpus", "2")
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_no_gpu_means_no_number():
    import torch
    if torch.cuda.is_available():
        return                                                  # on a GPU machine the benchmark itself covers this
    r = run("--steps", "1", "--warmup", "0")
    assert r.returncode == 3
    assert "no CPU fallback" in r.stderr and r.stdout.strip() == ""


import json

import pytest


@pytest.mark.gpu
@pytest.mark.parametrize("extra", [(), ("--scales", "rows"), ("--scales", "rows-single-read", "--scale-rule", "pow2"),
                                   ("--scales", "rows-single-read", "--scale-block", "128"), ("--calls", "plan")])
def test_bench_prints_one_json_line_with_the_agreed_fields(extra):
    """A short run on the small single-linear workload: one JSON line on stdout, with the fields the
    benchmark contract names, a roofline object for the longest fused launch and the oracle's timing."""
    r = run("--workload", "config0", "--steps", "3", "--warmup", "2", "--settle", "0", "--cpu-seconds", "0.5", *extra)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 2 and d["unit"] == "GB/s"
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["value"] > 0 and d["ms_per_step"] > 0 and "workload" in d["config"]
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12
    cpu = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0


def test_scale_block_needs_row_scales():
    r = run("--scale-block", "128")
    assert r.returncode == 2 and "--scales rows" in r.stderr and r.stdout.strip() == ""
