"""bench.py's command line, the shape of the one JSON line it prints, and the committed counter table it reads."""
import importlib.util
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_traffic_table_describes_the_launches_the_library_makes():
    """roofline.traffic comes from profiles/linear_mfma_traffic.md.  Every row names the kernel instance and grid its
    counters were read from; the launcher must still pick exactly that for the row's shape, or the figure is stale."""
    from paper_2506_04985_amd import binding as fptq
    rows = load_bench().read_traffic_table()
    assert "c5.gate_up" in rows, "the headline launch needs a row"
    for name, r in rows.items():
        kernel, workgroups, threads = fptq.fptq_linear_launch_plan(r["M"], r["N"], r["K"])
        assert (kernel, workgroups * threads) == (r["kernel"], r["grid"]), name
        algorithmic = r["N"] * r["K"] // 2 + r["M"] * r["K"] // 2 + 4 * r["N"] + 2 * r["M"] * r["N"]
        assert r["bytes"] >= 0.95 * algorithmic, name          # a launch cannot move less than its operands and its output
        assert r["fetch_scale"] > 0 and r["write_scale"] > 0
    head = rows["c5.gate_up"]
    assert (head["M"], head["N"], head["K"]) == (8192, 57344, 8192)


@pytest.mark.gpu
def test_json_line_has_the_contract_fields():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "1", "--no-decode", "--headline-only"],
                       capture_output=True, text=True, timeout=900)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["unit"] == "TOP/s" and d["higher_is_better"] is True and d["data"] == "synthetic"
    assert d["config"]["workload"].startswith("c5") and "model" not in d["config"] and d["config"]["tokens"] == 8192
    # value and ms_per_step describe the same timed region
    assert abs(d["value"] - d["config"]["ops_per_step"] / (d["ms_per_step"] * 1e-3) / 1e12) <= 0.01 * d["value"]
    r = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in r, key
    assert r["bound"] == "mfma" and r["peak"] == 5000.0 and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    assert 0.2 < r["frac"] < 1.0
    # the figure held against the roofline is the lower of the two regions' on the dominant launch
    assert r["achieved"] == min(r["own_activations"]["TOPS"], r["dense_int4_activations"]["TOPS"])
    assert r["ops_per_launch"] == 2 * 8192 * 57344 * 8192
    assert r["traffic"] is not None and "STALE" not in r["traffic_source"]      # the committed counter table is there and current
    assert r["traffic"] >= 0.95 * r["algorithmic_bytes_per_launch"]
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["sample"] and c["extrapolated"] is True
    assert "-O3" in c["compiler_flags"]
    assert set(d["configs"]) == {"c5"} and set(d["configs"]["c5"]["shapes"]) == {"qkv", "o", "gate_up", "down"}
