"""bench.py prints one JSON line with the agreed fields (a short run on the GPU)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_json_line():
    print("bench.py --steps 16 --warmup 2 --cpu-seconds 1", flush=True)
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "16", "--warmup", "2",
                        "--cpu-seconds", "1"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 16 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["unit"] == "TOP/s" and d["dtype"] == "int8" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["config"]["workload"] == "dit_xl2_256px_w8a8_m4096" and "model" not in d["config"]
    assert d["value"] > 100 and 0.01 < d["ms_per_step"] < 10
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["unit"] == "TOP/s" and rf["peak"] == 5000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9 and 0 < rf["frac"] < 1
    assert rf["traffic"] is None or rf["traffic"] > 1e6
    # the chip's own ceiling from the yardstick kernel: below the published peak, above what the path reaches
    assert rf["achieved"] < rf["measured_peak"] <= 5000.0 * 1.02
    rq = d["roofline_rotate_quant"]
    assert rq["bound"] == "hbm" and rq["achieved"] < rq["measured_peak"] <= 8000.0
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "TOP/s" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
