"""GPU: sample-wise use of the codec, as a pipeline stage would (Alg. 1 steps 4-5: send Q(a), de-quantize on arrival).
Runs of samples are encoded on several streams into self-contained streams, each is decoded as soon as its own encode
has completed -- in an order unrelated to the sample order -- and every stream and every decoded sample must equal what
the oracle gives for that run of samples taken as a tensor of its own."""
import sys

import numpy as np
import pytest

import workloads
from oracle import o32

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_gpu_parity import to_device  # noqa: E402


@pytest.fixture(scope="module")
def tahq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_01352_amd as t
    t.binding._load()
    return t


CASES = [
    # (config, shape, budget, samples per run): small ranking units; units of 65536 tiles (two-launch selection);
    # fp32 with a run length that does not divide the batch; single-pass encode (budget 4.0)
    (4, dict(batch=6, seq=96), 3.25, 1),
    (4, dict(batch=3, seq=512), 3.4, 1),
    (2, dict(batch=5, seq=40), 3.5, 2),
    (5, dict(batch=4, seq=30), 4.0, 3),
]


@pytest.mark.parametrize("index,shape,budget,per_run", CASES)
def test_runs_of_samples_on_several_streams_decoded_on_arrival(tahq, index, shape, budget, per_run):
    w, x = workloads.generate(index, **shape)
    print(f"[case] pipeline {w.name} {w.batch}x{w.seq}x{w.hidden} budget {budget} runs of {per_run}", file=sys.stderr,
          flush=True)
    cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget)
    x = np.ascontiguousarray(x).reshape(w.batch, w.seq, w.hidden)
    d_in = to_device(x)
    out_dtype = w.dtype
    out = torch.full((x.size,), -1, dtype=torch.int16 if out_dtype == tahq.BF16 else torch.int32, device="cuda")
    runs = [(first, min(per_run, w.batch - first)) for first in range(0, w.batch, per_run)]
    n_streams = 3
    enc_streams = [torch.cuda.Stream() for _ in range(n_streams)]
    dec_streams = [torch.cuda.Stream() for _ in range(2)]
    # a workspace per encode stream (runs on one stream follow each other), a packed buffer per run
    workspaces = [torch.full((max(tahq.tahq_samples_workspace_size(cfg, per_run), 16),), 0x3C, dtype=torch.uint8,
                             device="cuda") for _ in range(n_streams)]
    packed = [torch.full((tahq.tahq_samples_packed_size(cfg, count),), 0xA5, dtype=torch.uint8, device="cuda")
              for _, count in runs]
    torch.cuda.synchronize()
    done = []
    order = list(range(len(runs)))[::-1]             # enqueue the runs last-first: arrival order is not sample order
    for i in order:
        first, count = runs[i]
        s = enc_streams[i % n_streams]
        tahq.tahq_encode_samples(cfg, first, count, d_in, packed[i], workspaces[i % n_streams], s)
        ev = torch.cuda.Event()
        ev.record(s)
        done.append((i, ev))
    for j, (i, ev) in enumerate(done):
        first, count = runs[i]
        d = dec_streams[j % 2]
        d.wait_event(ev)                             # this run's stream has "arrived": decode it, nothing else is awaited
        tahq.tahq_decode_samples(cfg, first, count, packed[i], out, out_dtype, d)
    torch.cuda.synchronize()
    got_out = out.cpu().numpy().view(np.uint16 if out_dtype == tahq.BF16 else np.float32).reshape(x.shape)
    for i, (first, count) in enumerate(runs):
        xs = x[first:first + count]
        ocfg = o32.make_cfg(count, w.seq, w.hidden, w.tile, w.dtype, budget)
        want = o32.encode(ocfg, xs)
        assert np.array_equal(packed[i].cpu().numpy(), want), f"run {i}: stream differs from the oracle's"
        hdr = tahq.tahq_parse_header(want[:64].tobytes())
        assert (hdr.batch, hdr.seq, hdr.hidden) == (count, w.seq, w.hidden)
        want_out = o32.decode(ocfg, want, out_dtype).reshape(xs.shape)
        a, b = got_out[first:first + count], want_out
        if out_dtype == tahq.F32:
            a, b = a.view(np.uint32), b.view(np.uint32)
        assert np.array_equal(a, b), f"run {i}: decoded samples differ from the oracle's"


def test_sample_runs_argument_errors(tahq):
    import ctypes as C
    cfg = tahq.make_config(4, 8, 256, 64, tahq.BF16, 3.5)
    lib = tahq.binding._load()
    big = 1 << 30
    A, B_, W = 0x10000, 0x20000, 0x30000
    assert lib.tahq_encode_samples(C.byref(cfg), 4, 1, A, B_, big, W, big, None) == 2      # first sample outside
    assert lib.tahq_encode_samples(C.byref(cfg), 3, 2, A, B_, big, W, big, None) == 2      # run reaches outside
    assert lib.tahq_encode_samples(C.byref(cfg), 0, 0, A, B_, big, W, big, None) == 2
    assert lib.tahq_decode_samples(C.byref(cfg), 2, 3, A, big, B_, 1, None) == 2
    assert lib.tahq_encode_samples(C.byref(cfg), 1, 2, A, B_, 10, W, big, None) == 4       # packed buffer too small
    whole = tahq.make_config(4, 8, 256, 64, tahq.BF16, 3.5, scope=1)
    assert lib.tahq_encode_samples(C.byref(whole), 0, 1, A, B_, big, W, big, None) == 2    # samples are not independent
    assert tahq.tahq_samples_packed_size(whole, 1) == 0
    one = tahq.make_config(1, 8, 256, 64, tahq.BF16, 3.5)
    assert tahq.tahq_samples_packed_size(cfg, 1) == tahq.tahq_packed_size(one)
    assert tahq.tahq_samples_packed_size(cfg, 4) == tahq.tahq_packed_size(cfg)
    assert tahq.tahq_samples_packed_size(cfg, 5) == 0
