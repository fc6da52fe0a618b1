"""Host-side checks around the benchmark and the product/oracle separation.  CPU only."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_the_product_never_touches_the_oracle():
    # the package and the kernels' sources: no import of, link against or mention of the oracle's modules
    pkg = os.path.join(ROOT, "paper_2506_01352_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"\b(from|import)\s+oracle\b", text), f
                assert "libtahq_oracle" not in text and "libnaive_oracle" not in text and "tahq_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "include")):
        assert "oracle" not in open(os.path.join(ROOT, "include", f)).read(), f
    # bench.py reaches the oracles only inside its CPU-baseline legs
    src = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"from oracle import", src)]
    assert len(uses) == 2
    for pos in uses:
        head = src[:pos]
        func = head[head.rindex("\ndef "):]
        assert func.startswith("\ndef cpu_baseline") or "no_cpu_baseline" in func[-400:], func[:40]


def test_the_binding_fails_loudly_without_the_library():
    code = ("import paper_2506_01352_amd as t\n"
            "try:\n"
            "    t.tahq_version()\n"
            "except ImportError as e:\n"
            "    print('ImportError', e)\n")
    env = dict(os.environ, TAHQ_LIBRARY="/nonexistent/libtahq.so", PYTHONPATH=ROOT)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, cwd=ROOT)
    assert r.returncode == 0 and r.stdout.startswith("ImportError") and "no fallback" in r.stdout


def test_algorithmic_bytes_are_tensor_plus_stream():
    sys.path.insert(0, ROOT)
    import bench
    import workloads
    from oracle import o32
    w = workloads.CONFIGS[3]
    size = o32.packed_size(o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits))
    T = w.elements // w.tile
    alg = bench.algorithmic_bytes(w, size, T, True)
    assert alg["k_quant_pack"] == alg["k_decode"] == 2 * w.elements + size == 667680832
    assert alg["k_entropy"] == 2 * w.elements + 4 * T == 553648128


def test_stored_counter_readings_come_from_the_profile_summaries():
    # bench.py does not carry counter readings of its own: it parses profiles/hbm_traffic_*.md.  The streaming kernels'
    # measured traffic must stay within 2 % of their algorithmic bytes, and every kernel of a step must be listed.
    sys.path.insert(0, ROOT)
    import bench
    import workloads
    from oracle import o32
    per, step, src = bench.stored_traffic("hbm_traffic_cfg4_bf16_8x4096x8192_g64")
    assert src == "profiles/hbm_traffic_cfg4_bf16_8x4096x8192_g64.md"
    w = workloads.CONFIGS[3]
    size = o32.packed_size(o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits))
    alg = bench.algorithmic_bytes(w, size, w.elements // w.tile, True)
    for kernel in ("k_entropy", "k_quant_pack", "k_decode"):
        assert abs(per[kernel] / alg[kernel] - 1.0) < 0.02, kernel
    assert {"k_select_classify", "k_select_resolve"} <= set(per), sorted(per)
    assert step == sum(per.values()) and step > sum(alg.values())
    naive, _, nsrc = bench.stored_traffic("hbm_traffic_naive_cfg5_bf16_16x2048x5120_b8")
    assert nsrc and abs(naive["k_naive_encode"] / 503316544 - 1.0) < 0.02
    assert bench.stored_traffic("hbm_traffic_no_such_workload") == (None, None, None)
    # the vector-ALU readings of the same workload: instructions per tile and issue utilisation per kernel
    valu, vsrc = bench.stored_valu("valu_counters_cfg4_bf16_8x4096x8192_g64")
    assert vsrc == "profiles/valu_counters_cfg4_bf16_8x4096x8192_g64.md"
    for kernel in ("k_entropy", "k_quant_pack", "k_decode"):
        per_tile, pct = valu[kernel]
        assert 300 < per_tile < 1500 and 30 < pct < 130, (kernel, per_tile, pct)
    assert bench.stored_valu("valu_counters_no_such_workload") == (None, None)


def test_settling_steps_follow_the_requested_time():
    # bench.py runs plain untimed steps right before the timed region for about --settle-ms at the step time the warm-up
    # saw: at least --settle of them, at most 20000
    sys.path.insert(0, ROOT)
    import bench
    from types import SimpleNamespace as NS
    assert bench.settle_steps(NS(settle=10, settle_ms=150.0), 0.37) == int(150.0 / 0.37) + 1
    assert bench.settle_steps(NS(settle=10, settle_ms=0.0), 0.37) == 10
    assert bench.settle_steps(NS(settle=500, settle_ms=150.0), 0.37) == 500
    assert bench.settle_steps(NS(settle=10, settle_ms=150.0), 0.001) == 20000
    assert bench.settle_steps(NS(settle=10, settle_ms=150.0), 0.0) == 10
