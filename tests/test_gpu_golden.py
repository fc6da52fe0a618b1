"""GPU: the HIP path reproduces the stored digests of the oracles' outputs (tests/golden/) without calling
the oracles: stream, fp32 decode and bf16 decode of every stored case."""
import hashlib
import sys

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_golden import load_make_golden, stored_digests  # noqa: E402
from test_gpu_parity import to_device                      # noqa: E402


@pytest.fixture(scope="module")
def tahq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_01352_amd as t
    t.binding._load()
    return t


def digest(t):
    return hashlib.sha256(t.cpu().contiguous().view(torch.uint8).numpy().tobytes()).hexdigest()


def test_forward_codec_reproduces_stored_digests(tahq):
    mg, stored = load_make_golden(), stored_digests()
    for name, index, shape, kw in mg.FORWARD:
        print(f"[case] golden forward/{name}", file=sys.stderr, flush=True)
        w, x = workloads.generate(index, **shape)
        kw = dict(kw)
        cfg = tahq.make_config(w.batch, w.seq, w.hidden, kw.pop("tile", w.tile), w.dtype,
                               kw.pop("budget_bits", w.budget_bits), **kw)
        d_in = to_device(x)
        packed = torch.empty(tahq.tahq_packed_size(cfg), dtype=torch.uint8, device="cuda")
        ws = torch.empty(max(tahq.tahq_workspace_size(cfg), 16), dtype=torch.uint8, device="cuda")
        o32_ = torch.empty(x.size, dtype=torch.float32, device="cuda")
        o16 = torch.empty(x.size, dtype=torch.bfloat16, device="cuda")
        tahq.tahq_encode(cfg, d_in, packed, ws)
        tahq.tahq_decode(cfg, packed, o32_, tahq.F32)
        tahq.tahq_decode(cfg, packed, o16, tahq.BF16)
        torch.cuda.synchronize()
        assert (digest(packed), digest(o32_), digest(o16)) == stored["forward/" + name], name


def test_backward_compressor_reproduces_stored_digests(tahq):
    mg, stored = load_make_golden(), stored_digests()
    for name, index, shape, kw in mg.BACKWARD:
        print(f"[case] golden backward/{name}", file=sys.stderr, flush=True)
        w, x = workloads.generate(index, **shape)
        cfg = tahq.make_naive_config(w.batch, w.seq, w.hidden, w.dtype, kw["bits"], kw["scale"])
        d_in = to_device(x)
        packed = torch.empty(tahq.tahq_naive_packed_size(cfg), dtype=torch.uint8, device="cuda")
        o32_ = torch.empty(x.size, dtype=torch.float32, device="cuda")
        o16 = torch.empty(x.size, dtype=torch.bfloat16, device="cuda")
        tahq.tahq_naive_encode(cfg, d_in, packed)
        tahq.tahq_naive_decode(cfg, packed, o32_, tahq.F32)
        tahq.tahq_naive_decode(cfg, packed, o16, tahq.BF16)
        torch.cuda.synchronize()
        assert (digest(packed), digest(o32_), digest(o16)) == stored["backward/" + name], name
