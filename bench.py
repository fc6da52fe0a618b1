"""Benchmark of the TAH-Quant codec hot path on one MI355X.

One step = tahq_encode + tahq_decode of one micro-batch of synthetic activations that is
already resident in HBM.  Prints ONE JSON line: encode+decode GB/s of input activations, the
roofline of the dominant kernel (measured live with events on the launch stream) and the CPU
oracle's throughput on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--alloc-tile A] [--no-cpu-baseline]

`--codec naive [--bits 8] [--scale 16384]` measures the backward-pass fixed-point compressor instead
(default workload: configuration 5, the gradient-like tensor) and prints the same kind of line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs), each scaled by what
# the same counter reads for a plain copy kernel of known size; see profiles/ for the summaries.
TRAFFIC_BYTES = {
    ("cfg4_bf16_8x4096x8192_g64_b3.25", "k_quant_pack"): int((264287.7 * 2.0 + 127357.4) * 1024),
    ("cfg4_bf16_8x4096x8192_g64_b3.25", "k_entropy"): int((262221.1 * 2.0 + 16639.2) * 1024),
    ("cfg4_bf16_8x4096x8192_g64_b3.25", "k_decode"): int((65614.1 * 2.0 + 524452.6) * 1024),
    # the backward fixed-point compressor at its default 8 bits
    ("cfg5_bf16_16x2048x5120_g32_b4.0", "k_naive_encode"): int((163871.6 * 2.0 + 166564.4) * 1024),
    ("cfg5_bf16_16x2048x5120_g32_b4.0", "k_naive_decode"): int((83416.1 * 2.0 + 327685.7) * 1024),
}


# HBM bytes of ALL kernels of one encode+decode step (same counters, same scaling), for the share of the HBM peak that
# the whole path sustains: the three streaming kernels above plus prologue, two radix passes, segment counts, assignment.
STEP_TRAFFIC_BYTES = {
    "cfg4_bf16_8x4096x8192_g64_b3.25": 1975867392,
}


def algorithmic_bytes(w, packed_size, T, select):
    """Bytes each kernel must move per launch (per-element figures x elements of one launch)."""
    n, e = w.elements, w.bytes_per_element
    meta = packed_size - (w.tile // 8) * 3 * T            # rough: everything that is not 3-bit payload
    del meta
    return {
        # entropy kernel: reads the tensor once, writes one float per tile
        "k_entropy": n * e + 4 * T,
        # quantize+pack kernel: reads the tensor once, reads bit map + ranks, writes the stream
        "k_quant_pack": n * e + packed_size,
        # decode kernel: reads the stream once, writes the tensor once
        "k_decode": packed_size + n * e,
    }


def cpu_baseline(index, w, alloc_tile, low_bits, budget):
    """The oracle as it stands, single thread, on a bounded sample of the same workload."""
    import workloads
    from oracle import o32
    batch = max(1, min(w.batch, (150_000_000 + w.seq * w.hidden - 1) // (w.seq * w.hidden)))
    ws, x = workloads.generate(index, batch=batch, seq=w.seq, hidden=w.hidden)
    ocfg = o32.make_cfg(ws.batch, ws.seq, ws.hidden, w.tile, ws.dtype, budget, alloc_tile=alloc_tile, low_bits=low_bits)
    t0 = time.perf_counter()
    packed = o32.encode(ocfg, x)
    t1 = time.perf_counter()
    o32.decode(ocfg, packed, ws.dtype)
    t2 = time.perf_counter()
    nbytes = ws.elements * ws.bytes_per_element
    return {
        "value": nbytes / (t2 - t0) / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"first {batch} of {w.batch} samples of {w.name} ({ws.elements} elements): "
                  f"encode {t1 - t0:.2f} s + decode {t2 - t1:.2f} s",
    }


def naive_main(args):
    """tahq_naive_encode + tahq_naive_decode per step; both kernels are timed with events on every 4th step."""
    import numpy as np
    import torch
    import workloads
    import paper_2506_01352_amd as tahq

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    tahq.binding._load()
    index = args.config if args.config_given else 5
    w, x = workloads.generate(index)
    cfg = tahq.make_naive_config(w.batch, w.seq, w.hidden, w.dtype, args.bits, args.scale)
    size = tahq.tahq_naive_packed_size(cfg)
    if size == 0:
        print("bench.py: invalid --bits / --scale for the fixed-point compressor", file=sys.stderr)
        sys.exit(2)
    d_in = torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()
    packed = torch.empty(size, dtype=torch.uint8, device="cuda:0")
    out = torch.empty(w.elements, dtype=torch.bfloat16 if w.dtype else torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream()

    def step(ev=None):
        if ev:
            ev[0].record(stream)
        tahq.tahq_naive_encode(cfg, d_in, packed, stream)
        if ev:
            ev[1].record(stream)
        tahq.tahq_naive_decode(cfg, packed, out, w.dtype, stream)
        if ev:
            ev[2].record(stream)

    for _ in range(max(args.warmup, 1)):
        step()
    EVENT_EVERY = 4
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range((args.steps + EVENT_EVERY - 1) // EVENT_EVERY)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i // EVENT_EVERY] if i % EVENT_EVERY == 0 else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    nbytes = w.elements * w.bytes_per_element
    enc_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    dec_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    alg = nbytes + size                       # either kernel moves the tensor once and the stream once
    dominant, dom_ms = ("k_naive_encode", enc_ms) if enc_ms >= dec_ms else ("k_naive_decode", dec_ms)
    achieved = alg / (dom_ms * 1e-3) / 1e9
    out_line = {
        "metric": "fixed-point backward compressor: encode+decode GB/s of gradients on 1 MI355X",
        "value": nbytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "codec": "naive", "shape": [w.batch, w.seq, w.hidden],
                   "storage": "bf16" if w.dtype else "f32", "bits": args.bits, "scale": args.scale,
                   "out_dtype": "same as input"},
        "kernel_ms": {"k_naive_encode": enc_ms, "k_naive_decode": dec_ms},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": TRAFFIC_BYTES.get((w.name, dominant)) if args.bits == 8 else None,
                     "algorithmic_bytes_per_launch": alg,
                     "avg_launch_ms": dom_ms, "launches_timed": len(evs)},
    }
    if not args.no_cpu_baseline:
        from oracle import n32
        batch = max(1, min(w.batch, (150_000_000 + w.seq * w.hidden - 1) // (w.seq * w.hidden)))
        ws, xs = workloads.generate(index, batch=batch)
        ocfg = n32.make_cfg(ws.batch, ws.seq, ws.hidden, ws.dtype, args.bits, args.scale)
        c0 = time.perf_counter()
        p = n32.encode(ocfg, xs)
        c1 = time.perf_counter()
        n32.decode(ocfg, p, ws.dtype)
        c2 = time.perf_counter()
        out_line["cpu_baseline"] = {
            "value": ws.elements * ws.bytes_per_element / (c2 - c0) / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"first {batch} of {w.batch} samples of {w.name} ({ws.elements} elements): "
                      f"encode {c1 - c0:.2f} s + decode {c2 - c1:.2f} s"}
    print(json.dumps(out_line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=None, help="workload index 1..5 (default 4: the metric's config)")
    ap.add_argument("--codec", choices=("tahq", "naive"), default="tahq",
                    help="tahq: the forward activation codec (the metric); naive: the backward fixed-point compressor")
    ap.add_argument("--bits", type=int, default=8, help="--codec naive: code width, 2..16")
    ap.add_argument("--scale", type=float, default=16384.0, help="--codec naive: the pre-scale c")
    ap.add_argument("--alloc-tile", type=int, default=0,
                    help="allocation tile A in channels, a multiple of the tile width (default 0: A = G, the "
                         "metric's configuration)")
    ap.add_argument("--shape", type=str, default=None,
                    help="BxSxC: the chosen configuration's recipe at another shape, e.g. 2x1024x1600 for a "
                         "GPT2-XL-sized micro-batch (default: the configuration's own shape)")
    ap.add_argument("--tile", type=int, default=0, choices=(0, 8, 16, 32, 64, 128),
                    help="quantization tile G (default 0: the workload's own)")
    ap.add_argument("--low-bits", type=int, default=0, choices=(0, 2, 3),
                    help="the two code widths are lo and lo+1 (default 0: 3, the metric's INT3/INT4)")
    ap.add_argument("--budget", type=float, default=None,
                    help="mean payload bits per element (default: the workload's own; with --low-bits 2 the default "
                         "is the workload's minus one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of the input tensor (known size), so that a rocprofv3 --pmc "
                         "run of this command can scale FETCH_SIZE / WRITE_SIZE by what they read for it")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this codec runs on one GPU; nothing here shards across GPUs (use --gpus 1)", file=sys.stderr)
        sys.exit(2)
    args.config_given = args.config is not None
    if args.config is None:
        args.config = 4
    if args.codec == "naive":
        return naive_main(args)

    import numpy as np
    import torch
    import workloads
    import paper_2506_01352_amd as tahq

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    tahq.binding._load()

    if args.shape:
        B_, S_, C_ = (int(v) for v in args.shape.lower().split("x"))
        w, x = workloads.generate(args.config, batch=B_, seq=S_, hidden=C_)
    else:
        w, x = workloads.generate(args.config)
    if args.tile:
        import dataclasses
        w = dataclasses.replace(w, tile=args.tile)
    budget = args.budget if args.budget is not None else w.budget_bits - (1.0 if args.low_bits == 2 else 0.0)
    cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget, alloc_tile=args.alloc_tile,
                           low_bits=args.low_bits)
    if tahq.tahq_packed_size(cfg) == 0:
        print("bench.py: --alloc-tile must be a multiple of the tile width that divides the hidden size, and "
              "--budget must lie in [lo, lo+1]", file=sys.stderr)
        sys.exit(2)
    wide = args.alloc_tile not in (0, w.tile)
    d_in = torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()
    del x
    codec = tahq.Codec(cfg, device="cuda:0")          # decodes into the input dtype
    if args.copy_calibration:
        scratch = torch.empty_like(d_in)
        scratch.copy_(d_in)                           # one elementwise copy kernel: reads and writes the tensor once
        torch.cuda.synchronize()
        del scratch
    T = w.elements // w.tile
    k = tahq.tahq_k_per_unit(cfg)
    n_per_unit = w.seq * (w.hidden // (args.alloc_tile or w.tile))
    select = 0 < k < n_per_unit
    stream = torch.cuda.current_stream()

    P = tahq
    PHASES = [("prologue", P.PHASE_PROLOGUE), ("k_entropy", P.PHASE_ENTROPY), ("select", P.PHASE_SELECT),
              ("k_quant_pack", P.PHASE_QUANT)]

    def instrumented_step(events):
        """Every phase of tahq_encode as a call of its own, and tahq_decode, with an event between each."""
        for i, (_, mask) in enumerate(PHASES):
            events[i].record(stream)
            tahq.tahq_encode_phases(cfg, d_in, codec.packed, codec.workspace, mask, stream)
        events[4].record(stream)
        tahq.tahq_decode(cfg, codec.packed, codec.out, codec.out_dtype, stream)
        events[5].record(stream)

    # warm-up: instrumented, to find the dominant streaming kernel (an event costs a few microseconds of idle
    # GPU, so the timed region brackets that one kernel only)
    names = [n for n, _ in PHASES] + ["k_decode"]
    wev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(max(args.warmup, 1))]
    for ev in wev:
        instrumented_step(ev)
    torch.cuda.synchronize()
    warm_ms = {nm: float(np.median([e[i].elapsed_time(e[i + 1]) for e in wev])) for i, nm in enumerate(names)}
    alg = algorithmic_bytes(w, tahq.tahq_packed_size(cfg), T, select)
    # with A > G the entropy phase is several kernels (two passes over the tensor): not a roofline candidate
    streaming = {nm: warm_ms[nm] for nm in alg if (nm != "k_entropy" or (select and not wide))}
    dominant = max(streaming, key=streaming.get)

    # the timed step: tahq_encode and tahq_decode, with tahq_encode split only where the dominant kernel
    # needs its two events
    before = {"k_entropy": P.PHASE_PROLOGUE, "k_quant_pack": P.PHASE_PROLOGUE | P.PHASE_ENTROPY | P.PHASE_SELECT,
              "k_decode": P.PHASE_ALL}[dominant]
    own = {"k_entropy": P.PHASE_ENTROPY, "k_quant_pack": P.PHASE_QUANT, "k_decode": 0}[dominant]
    after = P.PHASE_ALL & ~(before | own)

    def step(e0, e1):
        tahq.tahq_encode_phases(cfg, d_in, codec.packed, codec.workspace, before, stream)
        if own:
            e0.record(stream)
            tahq.tahq_encode_phases(cfg, d_in, codec.packed, codec.workspace, own, stream)
            e1.record(stream)
            if after:
                tahq.tahq_encode_phases(cfg, d_in, codec.packed, codec.workspace, after, stream)
            tahq.tahq_decode(cfg, codec.packed, codec.out, codec.out_dtype, stream)
        else:
            e0.record(stream)
            tahq.tahq_decode(cfg, codec.packed, codec.out, codec.out_dtype, stream)
            e1.record(stream)

    # every EVENT_EVERY-th step of the timed region carries the two events (each costs a few microseconds of
    # idle GPU); the other steps are plain tahq_encode + tahq_decode
    EVENT_EVERY = 4
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range((args.steps + EVENT_EVERY - 1) // EVENT_EVERY)]

    def plain_step():
        tahq.tahq_encode(cfg, d_in, codec.packed, codec.workspace, stream)
        tahq.tahq_decode(cfg, codec.packed, codec.out, codec.out_dtype, stream)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % EVENT_EVERY == 0:
            step(*evs[i // EVENT_EVERY])
        else:
            plain_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    nbytes = w.elements * w.bytes_per_element
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    dom_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in evs]))
    achieved = alg[dominant] / (dom_ms * 1e-3) / 1e9
    # the stored counter readings belong to the metric's own configuration
    stock = not wide and args.low_bits in (0, 3) and budget == w.budget_bits and not args.tile and not args.shape
    traffic = TRAFFIC_BYTES.get((w.name, dominant)) if stock else None
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
        "algorithmic_bytes_per_launch": alg[dominant], "avg_launch_ms": dom_ms, "launches_timed": len(evs),
    }

    out = {
        "metric": "encode+decode GB/s of activations on 1 MI355X; % of HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "shape": [w.batch, w.seq, w.hidden], "storage": "bf16" if w.dtype else "f32",
                   "tile": w.tile, "alloc_tile": args.alloc_tile or w.tile, "budget_bits": budget,
                   "widths": [args.low_bits or 3, (args.low_bits or 3) + 1],
                   "out_dtype": "same as input"},
        "pct_hbm_peak_of_activation_rate": 100.0 * value / HBM_PEAK_GBS,
        # measured HBM traffic of every kernel of the step (rocprofv3 counters, see profiles/) over the step's time
        "pct_hbm_peak_of_measured_traffic": (100.0 * STEP_TRAFFIC_BYTES[w.name] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
                                             if stock and w.name in STEP_TRAFFIC_BYTES else None),
        "warmup_phase_ms": warm_ms,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, w, args.alloc_tile, args.low_bits, budget)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
