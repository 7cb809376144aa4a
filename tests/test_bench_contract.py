"""bench.py's contract: one GPU only, one JSON line with the agreed keys, the roofline and traffic figures read from
tracked files.  The CPU part needs no GPU; the GPU part runs bench.py as a child process on tiny settings."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def _run(args, timeout=400):
    return subprocess.run([sys.executable, BENCH] + args, capture_output=True, text=True, timeout=timeout, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    res = _run(["--gpus", "2"], timeout=120)
    assert res.returncode != 0
    assert "--gpus must be 1" in res.stderr
    assert not any(line.startswith("{") for line in res.stdout.splitlines())


def test_traffic_table_is_read_from_the_tracked_file():
    sys.path.insert(0, ROOT)
    import bench
    v = bench.measured_traffic("base", "dec_persist")
    assert v is not None and 3.0e8 < v < 1.0e9                   # above the algorithmic 339.7 MB, same order
    assert bench.measured_traffic("base", "no_such_kernel") is None
    table = open(os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")).read()
    assert "dec_persist" in table and "rocprofv3" in table       # the table names its source


def _json_line(stdout):
    lines = [l for l in stdout.splitlines() if l.startswith('{"metric"')]
    assert len(lines) == 1, stdout[-2000:]
    return json.loads(lines[0])


@pytest.mark.gpu
def test_default_mode_prints_one_line_with_the_agreed_keys():
    res = _run(["--steps", "1", "--warmup", "1", "--prof-passes", "1", "--no-cpu-baseline"])
    assert res.returncode == 0, res.stderr[-2000:]
    j = _json_line(res.stdout)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 1 and j["warmup"] == 1 and j["vs_baseline"] is None
    assert j["higher_is_better"] is True and j["data"] == "synthetic" and j["dtype"] == "f16"
    assert "workload" in j["config"] and "model" not in j["config"]
    assert j["value"] > 0 and j["ms_per_step"] > 0
    r = j["roofline"]
    assert r["bound"] in ("hbm", "mfma", "alu") and r["unit"] in ("GB/s", "TFLOP/s")
    assert r["peak"] in (8000.0, 2500.0) and 0.0 < r["frac"] < 1.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    assert r["traffic"] is None or r["traffic"] > 0
    # tokens/s is the whole pass: batch x generated tokens over the time of one pass
    assert abs(j["value"] - 32 * 32 / (j["ms_per_step"] * 1e-3)) / j["value"] < 1e-6


@pytest.mark.gpu
def test_phase_trace_mode_reports_every_phase_of_the_one_launch_step():
    res = _run(["--phase-trace", "--steps", "1"])
    assert res.returncode == 0, res.stderr[-2000:]
    j = _json_line(res.stdout)
    step = j["traced_steps"][0]
    assert set(step["phases"]) == {"qkv", "attention", "attention_output", "ffn1", "ffn2"}
    # unit counts of the ERNIE-base shape at batch 32: (strips / strips per unit) x row groups
    assert [step["phases"][k]["workgroups"] for k in ("qkv", "attention", "attention_output", "ffn1", "ffn2")] == [144, 192, 96, 192, 192]
    assert 100.0 < step["kernel_us"] < 2000.0
    assert abs(sum(step["phase_us_along_the_chain"].values()) - step["layer_us"]) < 0.1
    assert len(step["shader_clock_ghz_by_xcd"]) == 8 and all(0.5 < c < 3.0 for c in step["shader_clock_ghz_by_xcd"])
