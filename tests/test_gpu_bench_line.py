"""bench.py prints one JSON line that keeps its contract: the driver's fields, a roofline object whose
fraction cannot exceed 1 and whose effective rate is labelled as such, the live HBM anchor, and the CPU
baseline.  Run on the tiny workload in a child process (bench.py is a program, not a module)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_contract():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "tiny", "--steps", "3",
                          "--warmup", "1", "--cpu-rows", "500"], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [ln for ln in run.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "max_rel_err"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["config"]["workload"] == "tiny" and d["data"] == "synthetic" and d["higher_is_better"] is True
    assert d["value"] > 0 and d["ms_per_step"] > 0
    r = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "achieved_is", "frac_is", "hbm_anchor"):
        assert key in r, key
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert 0 < r["frac"] <= 1.0
    for table in ("table_2GiB", "table_8GiB"):
        a = r["hbm_anchor"][table]
        assert "skipped" not in a, a
        for leg in ("spmm_f32", "spmm_q8"):
            assert 0 < a[leg]["frac"] <= 1.0 and a[leg]["ms"] > 0
    c = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in c, key
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0
    e = d["max_rel_err"]
    assert e["plan_bit_exact"] and e["int8_codes_and_scales_bit_exact"]
    assert e["fp32_vs_oracle"] <= 1e-5 and e["int8_vs_oracle_dequantised"] <= 1e-2


def test_more_than_one_gpu_is_refused():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert run.returncode != 0 and "ONE GPU" in run.stderr
