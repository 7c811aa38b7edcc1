"""bench.py's output contract on a cut-down run: one JSON line with the fields the driver reads."""
import json
import os
import subprocess
import sys

import pytest

from conftest import ROOT

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]


def _run(*flags):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], capture_output=True, text=True,
                          cwd=ROOT, timeout=280)


def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    r = _run("--batch", "2", "--decode-steps", "6", "--steps", "1", "--warmup", "1", "--cpu-seconds", "1")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["unit"] == "tokens/s" and j["value"] > 0 and j["vs_baseline"] is None
    assert "workload" in j["config"] and "model" not in j["config"]
    rf = j["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9 and rf["launches"] == 40 * 6
    cb = j["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    assert j["speedup_vs_unpruned"] > 0


def test_bench_refuses_more_than_one_gpu():
    r = _run("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_bench_side_configurations_run():
    for flags in (["--lazy", "36:37-39"], ["--kv-format", "e4m3"], ["--attend-tile", "8"],
                  ["--layer-schedule", "pvtp", "--stride", "4", "--step-schedule", "exp", "--tau", "3"]):
        r = _run("--batch", "2", "--decode-steps", "4", "--steps", "1", "--warmup", "0", "--no-cpu-baseline",
                 "--no-unpruned", *flags)
        assert r.returncode == 0, (flags, r.stderr[-2000:])
        assert json.loads(r.stdout.splitlines()[-1])["value"] > 0
    r = _run("--batch", "2", "--decode-steps", "4", "--steps", "1", "--warmup", "0", "--no-cpu-baseline",
             "--no-unpruned", "--contiguous-tail")
    assert r.returncode == 0 and json.loads(r.stdout.splitlines()[-1])["config"]["tail"] == "contiguous", r.stderr[-2000:]


def test_bench_select_probe_runs():
    r = _run("--select-probe", "--batch", "2")
    assert r.returncode == 0, r.stderr[-2000:]
    rows = json.loads(r.stdout.splitlines()[-1])["rows"]
    assert {x["call"] for x in rows} == {"st3_select_topk", "st3_select_compact_layer", "st3_gather_rows"}
    assert all(x["us"] > 0 and x["bytes"] >= 0 for x in rows)
