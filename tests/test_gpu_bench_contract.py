"""The one JSON line bench.py prints: the keys the driver reads, the roofline of the dominant kernel and the oracle's
CPU rate, on the headline workload with a short timed region."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "3", "--warmup", "2"],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 3 and out["warmup"] == 2 and out["higher_is_better"] is True
    assert out["config"]["workload"] == "b32k_n8" and out["config"]["path"] == "materialized" and out["dtype"] == "bf16"
    assert out["value"] > 0 and out["ms_per_step"] > 0
    # value is pairs per second of the whole step: 8 rank calls of 4096 pairs
    assert out["value"] == pytest.approx(8 * 4096 / (out["ms_per_step"] * 1e-3), rel=1e-3)
    roof = out["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"], abs=1e-3) and 0.05 < roof["frac"] < 1.0
    assert roof["traffic"] is not None and roof["traffic"] > 5e8
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and "rank call" in cpu["sample"]


def test_smoke_entry_runs():
    """`__graft_entry__.smoke()`: one small call per path on cuda:0, checked against the oracle inside."""
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    entry.smoke()
