"""The benchmark's command-line contract: one JSON line with the agreed keys; more than one
GPU is refused with a message (this build has no collectives)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert p.returncode == 2
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_bad_degree_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--degree", "4"], capture_output=True,
                       text=True, timeout=120)
    assert p.returncode == 2 and "--degree" in p.stderr


@pytest.mark.gpu
def test_json_line_on_the_small_workload():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "1", "--steps", "4", "--warmup", "1",
                        "--graph"], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    r = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 4 and r["warmup"] == 1 and r["unit"] == "updates/s"
    assert r["config"]["workload"].startswith("cfg1") and r["vs_baseline"] is None and r["data"] == "synthetic"
    roof = r["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12 and 0 < roof["frac"] < 1
    assert roof["algorithmic_bytes_per_launch"] == 12 * 8 * 1_000_000
    cb = r["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    assert abs(r["value"] - 8 * 1_000_000 * 4 / (r["ms_per_step"] * 4e-3)) <= 1e-6 * r["value"]
    assert r["hip_graph"]["ms_per_step"] > 0


@pytest.mark.gpu
@pytest.mark.parametrize("flags", [
    ["--workload", "2", "--layout", "dense", "--unfused"],
    ["--workload", "2", "--layout", "probe", "--in-place"],
    ["--workload", "2", "--global-average", "--device-tables"],
    ["--workload", "2", "--degree", "5"],
    ["--workload", "4", "--overlap"],
    ["--workload", "4", "--graph", "--no-consensus"],
    ["--workload", "2", "--layout", "spread"],
    ["--workload", "2", "--layout", "interleaved"],
])
def test_variants_run_and_report(flags):
    """Every benchmark variant runs to completion and prints one well-formed line."""
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "1",
                        "--no-cpu-baseline", "--no-extra-legs"] + flags, capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    r = json.loads(p.stdout.strip())
    assert r["value"] > 1e10 and 0.2 < r["roofline"]["frac"] < 1.0, r
    assert r["config"]["workload"].startswith("cfg" + flags[1])


@pytest.mark.gpu
def test_default_form_reports_the_legs_it_is_read_against():
    """Without flags the line also carries the same step in place and on dense arrays, tables that are not one ring
    (the tiled kernel), the distance as a pass of its own, the reference streams (read-only, write-only, x + a g
    in the step kernel's access pattern) and the runtime's device copy."""
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "2", "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    r = json.loads(p.stdout.strip())
    for key in ("pitched_out_of_place", "pitched_in_place", "dense_out_of_place", "dense_in_place",
                "tiled_two_rings_pitched", "tiled_degree13_pitched", "consensus_alone_pitched", "spread_fresh_process",
                "dense_interleaved_fresh_process"):
        leg = r["legs"][key]
        assert 0.2 < leg["frac"] < 1.0 and leg["avg_launch_ms"] > 0 and leg["workload"].startswith("cfg2"), (key, leg)
    for block in ("reference_streams", "reference_streams_dense"):
        for key in ("read_x_and_g", "write_x_out", "axpy_x_plus_a_g"):
            assert 0.2 < r[block][key]["frac"] < 1.0, (block, key, r[block][key])
    assert r["reference_streams"]["axpy_x_plus_a_g"]["bytes_per_element"] == 12
    assert r["device_copy"]["achieved_GBps"] > 0
    assert r["roofline"]["target_frac"] == 0.80 and r["roofline"]["target_met"] == (r["roofline"]["frac"] >= 0.80)
    sp = r["cpu_baseline_sparse"]
    assert sp["single_thread"]["value"] > 0 and sp["all_cores"]["cores"] >= 1
    assert r["cpu_baseline"]["kind"] == "oracle"
