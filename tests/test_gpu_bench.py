"""GPU: bench.py prints one JSON line with the agreed fields, for the forward codec and the backward compressor."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "4", "--warmup", "2",
                        "--no-cpu-baseline"] + list(args), capture_output=True, text=True, timeout=280)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    return json.loads(lines[0])


def test_forward_bench_line():
    print("[case] bench.py default", file=sys.stderr, flush=True)
    d = run_bench()
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 4 and d["unit"] == "GB/s" and d["vs_baseline"] is None
    assert d["config"]["workload"].startswith("cfg4_") and d["data"] == "synthetic"
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9 and 0.05 < rf["frac"] < 1.0
    assert rf["kernel"] in ("k_entropy", "k_quant_pack", "k_decode") and rf["traffic"] > 0
    assert abs(d["value"] - 536870912 / (d["ms_per_step"] * 1e-3) / 1e9) < 1e-6 * d["value"]


def test_backward_bench_line():
    print("[case] bench.py --codec naive", file=sys.stderr, flush=True)
    d = run_bench("--codec", "naive")
    assert d["config"]["codec"] == "naive" and d["config"]["workload"].startswith("cfg5_")
    rf = d["roofline"]
    assert rf["kernel"] in ("k_naive_encode", "k_naive_decode") and 0.05 < rf["frac"] < 1.0
    assert rf["algorithmic_bytes_per_launch"] == 335544320 + 167772224
