"""GPU: tahq_encode_noalloc (the encoder on the library's built-in scratch, for callers that cannot allocate)
gives the bytes of tahq_encode on calls in a row that share the scratch, each smaller than the one before."""
import ctypes as C
import sys

import numpy as np
import pytest

import workloads
from oracle import o32

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def tahq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_01352_amd as t
    t.binding._load()
    return t


def _to_device(x):
    return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()


def test_noalloc_encode_matches_tahq_encode_on_calls_in_a_row(tahq):
    # (configuration, shape, budget): the first ranks units of 131072 tiles with the multi-launch selection (histograms,
    # per-workgroup partial histograms, keys and segment counts all live in the scratch), the second is a smaller tensor
    # on the same path, so whatever the first call left behind lies under and beyond what it uses, the third ranks
    # small units in a single launch, the last one (fp32, budget 4.0) needs no selection
    cases = [(4, dict(batch=2, seq=1024), 3.25), (4, dict(batch=1, seq=600), 3.4), (2, dict(batch=3, seq=50), 3.5),
             (1, dict(), 4.0)]
    stream = torch.cuda.current_stream()
    for index, shape, budget in cases:
        w, x = workloads.generate(index, **shape)
        print(f"[case] noalloc cfg{index} {w.batch}x{w.seq}x{w.hidden} budget {budget}", file=sys.stderr, flush=True)
        cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget)
        assert 0 < tahq.tahq_workspace_size(cfg) <= tahq.NOALLOC_MAX_WORKSPACE
        d_in = _to_device(x)
        size = tahq.tahq_packed_size(cfg)
        pad = 256
        raw = torch.full((size + 2 * pad,), 0xA5, dtype=torch.uint8, device="cuda")
        got = raw[pad:pad + size]
        want = torch.full((size,), 0x5A, dtype=torch.uint8, device="cuda")
        ws = torch.full((tahq.tahq_workspace_size(cfg),), 0x3C, dtype=torch.uint8, device="cuda")
        tahq.tahq_encode(cfg, d_in, want, ws, stream)
        tahq.tahq_encode_noalloc(cfg, d_in, got, stream)
        torch.cuda.synchronize()
        r = raw.cpu().numpy()
        assert (r[:pad] == 0xA5).all() and (r[pad + size:] == 0xA5).all(), "out-of-bounds write"
        assert torch.equal(got, want), f"cfg{index}: built-in scratch and caller's workspace give different streams"
        if x.size <= 1 << 22:
            ocfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget)
            assert np.array_equal(got.cpu().numpy(), o32.encode(ocfg, x)), f"cfg{index}: differs from the oracle"


def test_noalloc_encode_rejects_what_does_not_fit(tahq):
    # 16 samples of the metric's configuration need 56 MiB of scratch; the built-in buffer holds 32 MiB
    cfg = tahq.make_config(16, 4096, 8192, 64, tahq.BF16, 3.25)
    assert tahq.tahq_workspace_size(cfg) > tahq.NOALLOC_MAX_WORKSPACE
    lib = tahq.binding._load()
    # never-dereferenced addresses: the call fails in host validation
    assert lib.tahq_encode_noalloc(C.byref(cfg), 0x10000, 0x20000, 1 << 40, None) == 8
    assert "built-in" in tahq.tahq_status_string(8)
