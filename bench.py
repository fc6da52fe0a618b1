"""Benchmark of the TAH-Quant codec hot path on one MI355X.

One step = tahq_encode + tahq_decode of one micro-batch of synthetic activations that is already resident in HBM.
Prints ONE JSON line: encode+decode GB/s of input activations (and the share of the HBM peak, on the bytes the method must
move and on the bytes the counters saw), encode and decode times from events, the roofline of the dominant kernel
(measured live with events on the launch stream), a plain-copy ceiling measured in the same run, the decode time with
fp32 output, and the CPU oracle's throughput on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--alloc-tile A] [--no-cpu-baseline]

Timing: W instrumented warm-up steps, then plain untimed steps for about `--settle-ms` milliseconds (at least `--settle`
of them) right before the timed region: the GPU reaches its steady clocks only after some tens of milliseconds of load,
and a step measured before that is up to 15 % slower than the codec runs in a training job.  Then EXACTLY K steps
between two synchronizations.  `ms_per_step` is the wall-clock mean of those K steps; from 50 steps on it is the median of the K
per-step times taken with events at the step boundaries, and the wall-clock mean is reported beside it.

`--chunked` adds the pipeline rehearsal on one GPU (sample-wise encode on two streams, device -> pinned host -> device
copies standing in for the link, decode on arrival) next to the same trip for the whole tensor; `--graph` adds the
time per step of a captured HIP graph of encode + decode (small micro-batches are bound by launch latency).
`--codec naive [--bits 8] [--scale 16384]` measures the backward-pass fixed-point compressor instead (default
workload: configuration 5, the gradient-like tensor) and prints the same kind of line.
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
PROFILES = os.path.join(ROOT, "profiles")


def stored_traffic(stem):
    """HBM bytes per launch of every kernel of one step, as rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE measured them in the
    runs summarized under profiles/ (each counter scaled by what it reads for a plain copy of known size; the file
    states both factors).  Stored readings, not measured in this run: the file is named in the JSON line.
    `stem`: the summary's file name without ".md".
    Returns (dict kernel -> bytes, sum over the kernels of a step, file name) or (None, None, None)."""
    import re
    name = stem + ".md"
    path = os.path.join(PROFILES, name)
    if not os.path.exists(path):
        return None, None, None
    text = open(path).read()
    m = re.search(r"factor\s+of\s+([0-9.]+)\s+for\s+FETCH_SIZE.*?and\s+([0-9.]+)\s+for\s+WRITE_SIZE", text, re.S)
    if not m:
        return None, None, None
    f_scale, w_scale = float(m.group(1)), float(m.group(2))
    per_kernel = {}
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 3 and cells[0].startswith("k_"):
            try:
                fetch, write = float(cells[1]), float(cells[2])
            except ValueError:
                continue
            per_kernel[cells[0].split("<")[0]] = int((fetch * f_scale + write * w_scale) * 1024)
    if not per_kernel:
        return None, None, None
    return per_kernel, sum(per_kernel.values()), "profiles/" + name


def stored_valu(stem):
    """Vector-ALU instructions per tile and issue utilisation of every kernel of one step, from the rocprofv3 --pmc
    summary under profiles/ (stored readings, like stored_traffic).  Returns (dict kernel -> (instructions per tile,
    utilisation in per cent), file name) or (None, None)."""
    name = stem + ".md"
    path = os.path.join(PROFILES, name)
    if not os.path.exists(path):
        return None, None
    per_kernel = {}
    for line in open(path).read().splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 6 and cells[0].startswith("k_"):
            try:
                per_kernel[cells[0].split("<")[0]] = (float(cells[3]), float(cells[5].rstrip("% ")))
            except ValueError:
                continue
    return (per_kernel, "profiles/" + name) if per_kernel else (None, None)


def algorithmic_bytes(w, packed_size, T, select):
    """Bytes each kernel must move per launch (per-element figures x elements of one launch)."""
    del select
    n, e = w.elements, w.bytes_per_element
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
    batch = max(1, min(w.batch, (270_000_000 + w.seq * w.hidden - 1) // (w.seq * w.hidden)))
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


def settle_steps(args, step_ms_estimate):
    """Number of plain untimed steps to run right before the timed region: enough for --settle-ms at the step time the
    warm-up saw, at least --settle, at most 20000."""
    n = args.settle
    if args.settle_ms > 0 and step_ms_estimate > 0:
        n = max(n, int(args.settle_ms / step_ms_estimate) + 1)
    return min(n, 20000)


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

    wev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(max(args.warmup, 1))]
    for ev in wev:
        step(ev)
    torch.cuda.synchronize()
    warm_step_ms = float(np.median([e[0].elapsed_time(e[2]) for e in wev]))
    EVENT_EVERY = 4
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range((args.steps + EVENT_EVERY - 1) // EVENT_EVERY)]
    n_settle = settle_steps(args, warm_step_ms)
    for _ in range(n_settle):
        step()
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
    storage = "bf16" if w.dtype else "f32"
    naive_traffic, _, naive_src = stored_traffic(
        f"hbm_traffic_naive_cfg{index}_{storage}_{w.batch}x{w.seq}x{w.hidden}_b{args.bits}")
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
        "settle_steps": n_settle, "settle_ms": args.settle_ms,
        "kernel_ms": {"k_naive_encode": enc_ms, "k_naive_decode": dec_ms},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": naive_traffic.get(dominant) if naive_traffic else None, "traffic_source": naive_src,
                     "algorithmic_bytes_per_launch": alg,
                     "avg_launch_ms": dom_ms, "launches_timed": len(evs)},
    }
    if not args.no_cpu_baseline:
        from oracle import n32
        batch = max(1, min(w.batch, (270_000_000 + w.seq * w.hidden - 1) // (w.seq * w.hidden)))
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
    ap.add_argument("--settle", type=int, default=10,
                    help="least number of plain untimed steps right before the timed region")
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="plain untimed steps are run for about this long right before the timed region, so that the "
                         "timed steps see the GPU's steady clocks (0: only --settle steps)")
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
    ap.add_argument("--low-bits", type=int, default=0, choices=(0, 1, 2, 3, 4, 5, 6, 7),
                    help="the two code widths are lo and lo+1 (default 0: 3, the metric's INT3/INT4)")
    ap.add_argument("--budget", type=float, default=None,
                    help="mean payload bits per element (default: the workload's own, shifted by lo - 3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of the input tensor (known size), so that a rocprofv3 --pmc "
                         "run of this command can scale FETCH_SIZE / WRITE_SIZE by what they read for it")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the copy ceiling and the fp32-output decode (profiling runs: fewer kernels in the trace)")
    ap.add_argument("--chunked", action="store_true",
                    help="also rehearse the pipeline use on this one GPU: sample-wise encode on two streams, copies "
                         "through pinned host memory, decode on arrival, against the same trip for the whole tensor")
    ap.add_argument("--graph", action="store_true",
                    help="also time a captured HIP graph of encode + decode (a second figure; the eager one stays the metric)")
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
    low = args.low_bits or 3
    budget = args.budget if args.budget is not None else w.budget_bits + (low - 3)
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
    nbytes = w.elements * w.bytes_per_element
    packed_size = tahq.tahq_packed_size(cfg)

    def new_event():
        return torch.cuda.Event(enable_timing=True)

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
    wev = [[new_event() for _ in range(6)] for _ in range(max(args.warmup, 1))]
    for ev in wev:
        instrumented_step(ev)
    torch.cuda.synchronize()
    warm_ms = {nm: float(np.median([e[i].elapsed_time(e[i + 1]) for e in wev])) for i, nm in enumerate(names)}
    alg = algorithmic_bytes(w, packed_size, T, select)
    # with A > G the entropy phase is several kernels (two passes over the tensor): not a roofline candidate
    streaming = {nm: warm_ms[nm] for nm in alg if (nm != "k_entropy" or (select and not wide))}
    dominant = max(streaming, key=streaming.get)

    def plain_step():
        tahq.tahq_encode(cfg, d_in, codec.packed, codec.workspace, stream)
        tahq.tahq_decode(cfg, codec.packed, codec.out, codec.out_dtype, stream)

    # the timed step: tahq_encode and tahq_decode.  One event per step boundary (per-step times, their median);
    # every EVENT_EVERY-th step also carries an event between encode and decode, and tahq_encode is split there where
    # the dominant kernel needs its two events.
    before = {"k_entropy": P.PHASE_PROLOGUE, "k_quant_pack": P.PHASE_PROLOGUE | P.PHASE_ENTROPY | P.PHASE_SELECT,
              "k_decode": P.PHASE_ALL}[dominant]
    own = {"k_entropy": P.PHASE_ENTROPY, "k_quant_pack": P.PHASE_QUANT, "k_decode": 0}[dominant]
    after = P.PHASE_ALL & ~(before | own)

    def split_step(e0, e1, mid):
        tahq.tahq_encode_phases(cfg, d_in, codec.packed, codec.workspace, before, stream)
        if own:
            e0.record(stream)
            tahq.tahq_encode_phases(cfg, d_in, codec.packed, codec.workspace, own, stream)
            e1.record(stream)
            if after:
                tahq.tahq_encode_phases(cfg, d_in, codec.packed, codec.workspace, after, stream)
            mid.record(stream)
            tahq.tahq_decode(cfg, codec.packed, codec.out, codec.out_dtype, stream)
        else:
            mid.record(stream)
            e0.record(stream)
            tahq.tahq_decode(cfg, codec.packed, codec.out, codec.out_dtype, stream)
            e1.record(stream)

    EVENT_EVERY = 4
    n_split = (args.steps + EVENT_EVERY - 1) // EVENT_EVERY
    evs = [(new_event(), new_event(), new_event()) for _ in range(n_split)]
    bounds = [new_event() for _ in range(args.steps + 1)]

    n_settle = settle_steps(args, sum(warm_ms.values()))
    for _ in range(n_settle):
        plain_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        bounds[i].record(stream)
        if i % EVENT_EVERY == 0:
            split_step(*evs[i // EVENT_EVERY])
        else:
            plain_step()
    bounds[args.steps].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    wall_ms = (t1 - t0) * 1e3 / args.steps
    step_ms = [bounds[i].elapsed_time(bounds[i + 1]) for i in range(args.steps)]
    median_ms = float(np.median(step_ms))
    ms_per_step = median_ms if args.steps >= 50 else wall_ms
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    encode_ms = float(np.median([bounds[EVENT_EVERY * j].elapsed_time(evs[j][2]) for j in range(n_split)]))
    decode_ms = float(np.median([evs[j][2].elapsed_time(bounds[EVENT_EVERY * j + 1]) for j in range(n_split)]))
    dom_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1, _ in evs]))
    achieved = alg[dominant] / (dom_ms * 1e-3) / 1e9

    # a plain device copy of the input tensor and a plain fill of as many bytes, right after the timed region (the GPU
    # is at its steady clocks): what this machine's HBM gives kernels that only move bytes
    copy_gbs = fill_gbs = None
    if not args.no_extras:
        scratch = torch.empty_like(d_in)
        cev = [(new_event(), new_event(), new_event()) for _ in range(6)]
        for a, b, c in cev:
            a.record(stream)
            scratch.copy_(d_in)
            b.record(stream)
            scratch.fill_(1)
            c.record(stream)
        torch.cuda.synchronize()
        copy_gbs = 2 * nbytes / (min(a.elapsed_time(b) for a, b, _ in cev[1:]) * 1e-3) / 1e9
        fill_gbs = nbytes / (min(b.elapsed_time(c) for _, b, c in cev[1:]) * 1e-3) / 1e9
        del scratch

    # decode into fp32 (twice the output bytes): a second figure, outside the timed region
    decode_f32_ms = None
    if not args.no_extras:
        out32 = torch.empty(w.elements, dtype=torch.float32, device="cuda:0")
        fev = [(new_event(), new_event()) for _ in range(6)]
        for a, b in fev:
            a.record(stream)
            tahq.tahq_decode(cfg, codec.packed, out32, tahq.F32, stream)
            b.record(stream)
        torch.cuda.synchronize()
        decode_f32_ms = float(np.median([a.elapsed_time(b) for a, b in fev[1:]]))
        del out32

    # the stored counter readings belong to the metric's own configuration
    stock = not wide and low == 3 and budget == w.budget_bits and not args.tile and not args.shape
    storage = "bf16" if w.dtype else "f32"
    stem = f"cfg{args.config}_{storage}_{w.batch}x{w.seq}x{w.hidden}_g{w.tile}"
    traffic, step_traffic, traffic_src = stored_traffic("hbm_traffic_" + stem) if stock else (None, None, None)
    valu, valu_src = stored_valu("valu_counters_" + stem) if stock else (None, None)
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS, "traffic": traffic.get(dominant) if traffic else None,
        "traffic_source": traffic_src,
        "algorithmic_bytes_per_launch": alg[dominant], "avg_launch_ms": dom_ms, "launches_timed": len(evs),
        # the co-bound: vector-ALU instructions per tile and issue utilisation of the same kernel (stored readings)
        "valu_instructions_per_tile": valu[dominant][0] if valu and dominant in valu else None,
        "valu_issue_utilisation_pct": valu[dominant][1] if valu and dominant in valu else None,
        "valu_source": valu_src,
    }
    # bytes the method must move: the tensor in, the stream out, the stream in, the tensor out
    must_move = 2 * nbytes + 2 * packed_size

    out = {
        "metric": "encode+decode GB/s of activations on 1 MI355X; % of HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "shape": [w.batch, w.seq, w.hidden], "storage": storage,
                   "tile": w.tile, "alloc_tile": args.alloc_tile or w.tile, "budget_bits": budget,
                   "widths": [low, low + 1], "out_dtype": "same as input"},
        "ms_per_step_is": "median of per-step event times" if args.steps >= 50 else "wall-clock mean",
        "ms_per_step_wall": wall_ms, "ms_per_step_median": median_ms, "settle_steps": n_settle, "settle_ms": args.settle_ms,
        "encode_ms": encode_ms, "decode_ms": decode_ms,
        "decode_f32_out_ms": decode_f32_ms,
        "value_f32_out": (nbytes / ((encode_ms + decode_f32_ms) * 1e-3) / 1e9) if decode_f32_ms else None,
        "copy_ceiling_gbs": copy_gbs, "fill_ceiling_gbs": fill_gbs,
        "pct_hbm_peak_of_activation_rate": 100.0 * value / HBM_PEAK_GBS,
        # (B) the bytes the method must move over the step's time; (A) the bytes the counters saw for every kernel
        # of the step (stored rocprofv3 readings, see traffic_source) over the step's time
        "pct_hbm_peak_algorithmic": 100.0 * must_move / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "pct_hbm_peak_of_measured_traffic": (100.0 * step_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
                                             if step_traffic else None),
        "step_traffic_bytes": step_traffic,
        "warmup_phase_ms": warm_ms,
        "roofline": roofline,
    }
    if args.graph:
        out["graph"] = graph_replay(tahq, torch, np, cfg, codec, d_in, args.steps, nbytes, max(5, n_settle))
    if args.chunked:
        out["chunked"] = chunked_loopback(tahq, torch, np, cfg, codec, d_in, w)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, w, args.alloc_tile, args.low_bits, budget)
    print(json.dumps(out))


def graph_replay(tahq, torch, np, cfg, codec, d_in, steps, nbytes, settle):
    """encode + decode captured once into a HIP graph and replayed `steps` times: what a caller pays per step when the
    launches are taken off the host (matters for micro-batches of the size the paper trains with)."""
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            tahq.tahq_encode(cfg, d_in, codec.packed, codec.workspace, s)
            tahq.tahq_decode(cfg, codec.packed, codec.out, codec.out_dtype, s)
        for _ in range(settle):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / steps
    return {"ms_per_step": ms, "value": nbytes / (ms * 1e-3) / 1e9, "unit": "GB/s", "replays": steps}


def chunked_loopback(tahq, torch, np, cfg, codec, d_in, w, reps=5):
    """Pipeline rehearsal on one GPU (Alg. 1 steps 4-5).  The link between two stages is played by a copy of the stream
    to pinned host memory and back.  (a) whole tensor: encode, copy out, copy back, decode, one after the other;
    (b) sample-wise: every sample is encoded on one of two streams into a stream of its own, copied out and back on a
    copy stream as soon as its encode is done, and decoded on a third stream as soon as it is back."""
    size = tahq.tahq_packed_size(cfg)
    host = torch.empty(size, dtype=torch.uint8, pin_memory=True)
    back = torch.empty(size, dtype=torch.uint8, device="cuda:0")
    main = torch.cuda.current_stream()

    def whole():
        tahq.tahq_encode(cfg, d_in, codec.packed, codec.workspace, main)
        host.copy_(codec.packed, non_blocking=True)
        back.copy_(host, non_blocking=True)
        tahq.tahq_decode(cfg, back, codec.out, codec.out_dtype, main)

    B = cfg.batch
    ssize = tahq.tahq_samples_packed_size(cfg, 1)
    wsize = max(tahq.tahq_samples_workspace_size(cfg, 1), 16)
    enc = [torch.cuda.Stream(), torch.cuda.Stream()]
    cpy, dec = torch.cuda.Stream(), torch.cuda.Stream()
    ws = [torch.empty(wsize, dtype=torch.uint8, device="cuda:0") for _ in enc]
    dev = [torch.empty(ssize, dtype=torch.uint8, device="cuda:0") for _ in range(B)]
    hst = [torch.empty(ssize, dtype=torch.uint8, pin_memory=True) for _ in range(B)]
    bck = [torch.empty(ssize, dtype=torch.uint8, device="cuda:0") for _ in range(B)]

    def chunked():
        for s in enc + [cpy, dec]:
            s.wait_stream(main)
        for i in range(B):
            e = enc[i % 2]
            tahq.tahq_encode_samples(cfg, i, 1, d_in, dev[i], ws[i % 2], e)
            ev = torch.cuda.Event()
            ev.record(e)
            cpy.wait_event(ev)
            with torch.cuda.stream(cpy):
                hst[i].copy_(dev[i], non_blocking=True)
                bck[i].copy_(hst[i], non_blocking=True)
            ev2 = torch.cuda.Event()
            ev2.record(cpy)
            dec.wait_event(ev2)
            tahq.tahq_decode_samples(cfg, i, 1, bck[i], codec.out, codec.out_dtype, dec)
        main.wait_stream(dec)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        return float(np.median(ts))

    whole_ms = timed(whole)
    chunk_ms = timed(chunked)
    # codec alone, sample-wise on the two streams (no copies)
    def chunk_codec_only():
        for s in enc + [dec]:
            s.wait_stream(main)
        for i in range(B):
            e = enc[i % 2]
            tahq.tahq_encode_samples(cfg, i, 1, d_in, dev[i], ws[i % 2], e)
            ev = torch.cuda.Event()
            ev.record(e)
            dec.wait_event(ev)
            tahq.tahq_decode_samples(cfg, i, 1, dev[i], codec.out, codec.out_dtype, dec)
        main.wait_stream(dec)
    codec_ms = timed(chunk_codec_only)
    return {"whole_tensor_ms": whole_ms, "sample_wise_ms": chunk_ms, "sample_wise_codec_only_ms": codec_ms,
            "stream_bytes": size, "samples": B, "link": "device -> pinned host -> device",
            "reps": reps}


if __name__ == "__main__":
    main()
