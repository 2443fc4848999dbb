"""bench.py's one-line JSON contract, on a shortened run (2 resident layers, 40 steps)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--layers", "2", "--steps", "40", "--warmup", "8"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 40 and d["warmup"] == 8 and d["unit"] == "GB/s" and d["vs_baseline"] is None
    assert d["higher_is_better"] is True and d["data"] == "synthetic" and "workload" in d["config"]
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3 and 0.05 < roof["frac"] < 1.0
    assert abs(d["value"] - d["config"]["kv_bytes_per_step"] / (d["ms_per_step"] * 1e-3) / 1e9) < 0.01 * d["value"]
    assert d["config"]["preroll_steps"] > 0
    others = d["config"]["other_configs"]
    assert set(others) == {"configs[0]", "configs[1]", "configs[2]", "configs[4]"}
    assert others["configs[1]"]["decode_step_us"] > 0 and others["configs[4]"]["quantize_tok_s_back_to_back"] > 0
    assert len(others["configs[2]"]["points"]) == 15 and others["configs[0]"]["decode_step_us_back_to_back"] > 0
    qr = roof["quantize"]
    assert qr["bound"] == "hbm" and 0.05 < qr["frac"] < 1.0 and abs(qr["frac"] - qr["achieved"] / qr["peak"]) < 1e-3
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    assert cpu["planes_byte_identical"] is True and cpu["parity_max_rel_err_vs_oracle"] < 2e-3


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "single-GPU" in r.stderr
