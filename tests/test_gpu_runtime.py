"""GPU: how the library behaves under the callers it is meant for -- several host threads on their own streams,
and a captured HIP graph replayed in a loop (the library only enqueues kernels, allocates nothing and keeps no
state between calls, so both must give the oracle's bytes)."""
import sys
import threading

import numpy as np
import pytest

import workloads
from oracle import n32, o32

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


def test_two_host_threads_on_their_own_streams(tahq):
    cases = [(2, dict(batch=2, seq=40)), (4, dict(batch=2, seq=36))]
    results, errors = {}, []

    def worker(slot, index, shape):
        try:
            torch.cuda.set_device(0)
            w, x = workloads.generate(index, **shape)
            cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.4)
            codec = tahq.Codec(cfg, out_dtype=tahq.F32)
            d_in = to_device(x)
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            outs = []
            for _ in range(6):
                codec.encode(d_in, stream=s)
                codec.decode(stream=s)
                s.synchronize()
                outs.append((codec.packed.cpu().numpy().copy(), codec.out.cpu().numpy().copy()))
            results[slot] = (w, x, outs)
        except Exception as e:                      # reported by the main thread
            errors.append((slot, repr(e)))

    print("[case] two host threads", file=sys.stderr, flush=True)
    threads = [threading.Thread(target=worker, args=(i, idx, shape)) for i, (idx, shape) in enumerate(cases)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not errors, errors
    assert len(results) == 2
    for slot, (w, x, outs) in results.items():
        ocfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.4)
        want = o32.encode(ocfg, x)
        want_out = o32.decode(ocfg, want, o32.F32)
        for packed, out in outs:
            assert np.array_equal(packed, want), slot
            assert np.array_equal(out.view(np.uint32), want_out.view(np.uint32)), slot


def test_captured_graph_replays_give_the_eager_bytes(tahq):
    # encode + decode of the forward codec and of the backward compressor captured once, replayed on new inputs,
    # with eager work and synchronizations between the replays; every replay is checked against the oracle
    w, x0 = workloads.generate(4, batch=2, seq=48)
    cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
    ocfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
    ncfg = tahq.make_naive_config(w.batch, w.seq, w.hidden, w.dtype, 8, 64.0)
    nocfg = n32.make_cfg(w.batch, w.seq, w.hidden, w.dtype, 8, 64.0)
    codec = tahq.Codec(cfg)
    d_in = to_device(x0)
    npacked = torch.empty(tahq.tahq_naive_packed_size(ncfg), dtype=torch.uint8, device="cuda")
    nout = torch.empty(x0.size, dtype=torch.bfloat16, device="cuda")

    def enqueue(stream):
        codec.encode(d_in, stream=stream)
        codec.decode(stream=stream)
        tahq.tahq_naive_encode(ncfg, d_in, npacked, stream)
        tahq.tahq_naive_decode(ncfg, npacked, nout, tahq.BF16, stream)

    enqueue(torch.cuda.current_stream())            # eager warm-up: also fills the library's launch-size caches
    torch.cuda.synchronize()
    print("[case] graph capture", file=sys.stderr, flush=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue(torch.cuda.current_stream())
    rng = np.random.default_rng(11)
    for rep in range(4):
        print(f"[case] graph replay {rep}", file=sys.stderr, flush=True)
        xf = workloads.bf16_bits_to_f32(x0) * np.float32(1.0 + 0.25 * rep)
        xf[rep % 2, rng.integers(0, w.seq), :] = 0.0
        x = workloads.f32_to_bf16_bits(xf)
        d_in.copy_(to_device(x))
        codec.packed.fill_(0x77)                    # eager work between the replays
        npacked.fill_(0x77)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = o32.encode(ocfg, x)
        assert np.array_equal(codec.packed.cpu().numpy(), want), rep
        got = codec.out.cpu().view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got, o32.decode(ocfg, want, w.dtype)), rep
        nwant = n32.encode(nocfg, x)
        assert np.array_equal(npacked.cpu().numpy(), nwant), rep
        assert np.array_equal(nout.cpu().view(torch.int16).numpy().view(np.uint16), n32.decode(nocfg, nwant, n32.BF16)), rep
