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
    # four steps: the wall-clock mean is the figure; encode and decode from events, the copy ceiling and the fp32-output
    # decode measured in the same run, both shares of the HBM peak
    assert d["ms_per_step_is"] == "wall-clock mean" and d["ms_per_step"] == d["ms_per_step_wall"]
    assert 0 < d["decode_ms"] < d["encode_ms"] < d["ms_per_step"] * 1.5
    assert d["decode_f32_out_ms"] > d["decode_ms"] and 1000 < d["copy_ceiling_gbs"] < 8000
    assert 1000 < d["fill_ceiling_gbs"] < 8000 and d["settle_steps"] >= 10
    assert rf["valu_instructions_per_tile"] > 100 and 0 < rf["valu_issue_utilisation_pct"] < 130
    assert 0 < d["pct_hbm_peak_algorithmic"] < d["pct_hbm_peak_of_measured_traffic"] < 100
    assert rf["traffic_source"].startswith("profiles/hbm_traffic_cfg4_")


def test_forward_bench_line_graph_and_sample_wise_rehearsal():
    print("[case] bench.py --graph --chunked on a small shape", file=sys.stderr, flush=True)
    d = run_bench("--shape", "4x256x2048", "--budget", "3.5", "--graph", "--chunked")
    assert d["graph"]["ms_per_step"] > 0 and d["graph"]["replays"] == 4
    c = d["chunked"]
    assert c["samples"] == 4 and c["whole_tensor_ms"] > 0 and c["sample_wise_ms"] > 0
    assert d["roofline"]["traffic"] is None and d["pct_hbm_peak_of_measured_traffic"] is None


def test_backward_bench_line():
    print("[case] bench.py --codec naive", file=sys.stderr, flush=True)
    d = run_bench("--codec", "naive")
    assert d["config"]["codec"] == "naive" and d["config"]["workload"].startswith("cfg5_")
    rf = d["roofline"]
    assert rf["kernel"] in ("k_naive_encode", "k_naive_decode") and 0.05 < rf["frac"] < 1.0
    assert rf["algorithmic_bytes_per_launch"] == 335544320 + 167772224
