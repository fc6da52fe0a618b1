"""GPU parity of the backward-pass fixed-point compressor (through the C ABI) against its CPU oracle:
the stream byte for byte, decoded fp32 and bf16 output bit for bit."""
import sys

import numpy as np
import pytest

import workloads
from oracle import n32

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_gpu_parity import Guarded, to_device, first_diff  # noqa: E402


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def tahq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_01352_amd as t
    t.binding._load()          # fail loudly if the HIP library is missing
    return t


def check_case(tahq, x, B, S, Cc, dtype, bits, scale, out_dtypes=(0, 1)):
    x = np.ascontiguousarray(x).reshape(B, S, Cc)
    cfg = tahq.make_naive_config(B, S, Cc, dtype, bits, scale)
    ocfg = n32.make_cfg(B, S, Cc, dtype, bits, scale)
    d_in = to_device(x)
    packed = Guarded(tahq.tahq_naive_packed_size(cfg))
    tahq.tahq_naive_encode(cfg, d_in, packed.view)
    outs = {}
    for od in out_dtypes:
        outs[od] = Guarded((4 if od == tahq.F32 else 2) * x.size)
        tahq.tahq_naive_decode(cfg, packed.view, outs[od].view, od)
    torch.cuda.synchronize()
    packed.check()
    want = n32.encode(ocfg, x)
    got = packed.view.cpu().numpy()
    assert np.array_equal(got[:64], want[:64]), "header differs"
    d = first_diff(got, want)
    assert d is None, f"payload differs at byte {d} (element {(d - 64) * 8 // bits}): got {got[d]:#x}, want {want[d]:#x}"
    for od, g in outs.items():
        g.check()
        want_out = n32.decode(ocfg, want, od)
        o = g.view.cpu().numpy().view(np.float32 if od == tahq.F32 else np.uint16)
        cmp = np.uint32 if od == tahq.F32 else np.uint16
        assert np.array_equal(o.view(cmp), want_out.view(cmp)), f"decoded output (dtype {od}) differs at {first_diff(o.view(cmp), want_out.view(cmp))}"


@pytest.mark.parametrize("bits", tuple(range(2, 17)))
@pytest.mark.parametrize("dtype_name", ("f32", "bf16"))
def test_every_width_and_dtype_several_workgroups_and_a_ragged_tail(tahq, bits, dtype_name):
    # a workgroup handles 256 chunks of 32 elements: 3 full workgroups plus 37 chunks, rows that straddle them
    Cc = 96
    S = (3 * 256 + 37) * 32 // Cc
    rng = np.random.default_rng(40 + bits)
    hi = 2.0 ** (bits - 1)
    x = (rng.standard_normal((1, S, Cc)) * hi * 0.4).astype(np.float32)
    x[0, ::5, 7] *= 6.0                                            # beyond the range: clamps
    x[0, 3, :] = (rng.integers(-int(hi) - 2, int(hi) + 2, size=Cc) + 0.5).astype(np.float32)   # exact ties
    x[0, 4, :] = 0.0
    x[0, 6, :8] = [np.inf, -np.inf, np.nan, -0.0, 1e30, -1e30, 0.5, -0.5]
    bf16 = dtype_name == "bf16"
    with np.errstate(all="ignore"):
        xin = workloads.f32_to_bf16_bits(x) if bf16 else x
    for scale in (1.0, 0.37):
        _say(f"[case] naive bits={bits} {dtype_name} scale={scale} shape=1x{S}x{Cc}")
        check_case(tahq, xin, 1, S, Cc, tahq.BF16 if bf16 else tahq.F32, bits, scale)


@pytest.mark.parametrize("bits,scale", [(4, 2.0 ** 9), (6, 2.0 ** 12), (8, 2.0 ** 14), (10, 2.0 ** 16), (8, 12345.678)])
def test_gradient_like_workload(tahq, bits, scale):
    w, x = workloads.generate(5, batch=3, seq=33)
    _say(f"[case] naive {w.name} 3x33x{w.hidden} bits={bits} scale={scale}")
    check_case(tahq, x, w.batch, w.seq, w.hidden, w.dtype, bits, scale)
    w2, x2 = workloads.generate(2, batch=2, seq=40)
    check_case(tahq, x2 * np.float32(2.0 ** -10), w2.batch, w2.seq, w2.hidden, w2.dtype, bits, scale)


def test_tiny_tensors(tahq):
    rng = np.random.default_rng(2)
    for B, S, Cc in ((1, 1, 32), (1, 1, 64), (2, 1, 32), (1, 3, 1600)):
        x = (rng.standard_normal((B, S, Cc)) * 20).astype(np.float32)
        for bits in (2, 7, 8, 16):
            _say(f"[case] naive tiny {B}x{S}x{Cc} bits={bits}")
            check_case(tahq, x, B, S, Cc, tahq.F32, bits, 1.5)


def test_full_size_gradient_tensor_sampled(tahq):
    # configuration 5 at full size (16 x 2048 x 5120 bf16), 8 bits: the oracle checks the first and last samples
    # and a window in the middle byte for byte
    w, x = workloads.generate(5)
    bits, scale = 8, 2.0 ** 14
    _say(f"[case] naive full size {w.name}")
    cfg = tahq.make_naive_config(w.batch, w.seq, w.hidden, w.dtype, bits, scale)
    d_in = to_device(x)
    packed = torch.empty(tahq.tahq_naive_packed_size(cfg), dtype=torch.uint8, device="cuda")
    out = torch.empty(x.size, dtype=torch.bfloat16, device="cuda")
    tahq.tahq_naive_encode(cfg, d_in, packed)
    tahq.tahq_naive_decode(cfg, packed, out, tahq.BF16)
    torch.cuda.synchronize()
    got = packed.cpu().numpy()
    got_out = out.cpu().view(torch.int16).numpy().view(np.uint16)
    per = w.seq * w.hidden
    flat = x.reshape(-1)
    for b0, nb in ((0, 1), (w.batch // 2, 1), (w.batch - 1, 1)):
        sl = flat[b0 * per:(b0 + nb) * per]
        ocfg = n32.make_cfg(nb, w.seq, w.hidden, w.dtype, bits, scale)
        want = n32.encode(ocfg, sl)
        lo = 64 + b0 * per * bits // 8
        assert np.array_equal(got[lo:lo + nb * per * bits // 8], want[64:]), f"sample {b0}"
        assert np.array_equal(got_out[b0 * per:(b0 + nb) * per], n32.decode(ocfg, want, n32.BF16)), f"sample {b0}"


def _random_naive_cases(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        out.append(dict(B=int(rng.choice([1, 2, 5])), S=int(rng.choice([1, 7, 64, 333])), Cc=32 * int(rng.choice([1, 3, 16, 50, 129])),
                        dtype=int(rng.integers(0, 2)), bits=int(rng.integers(2, 17)),
                        scale=float(rng.choice([1.0, 2.0 ** 10, 2.0 ** -4, 3.3, 1e4, 7e-3])), seed=int(rng.integers(0, 2 ** 31))))
    return out


@pytest.mark.parametrize("c", _random_naive_cases(60, seed=99), ids=lambda c: "{B}x{S}x{Cc}_d{dtype}_b{bits}".format(**c))
def test_random_configurations_bit_exact(tahq, c):
    rng = np.random.default_rng(c["seed"])
    span = 2.0 ** (c["bits"] - 1) / c["scale"]
    x = (rng.standard_normal((c["B"], c["S"], c["Cc"])) * span * 0.5).astype(np.float32)
    x[..., ::11] *= 4.0                                              # part of it beyond the range
    x[..., 5::13] = 0.0
    xin = workloads.f32_to_bf16_bits(x) if c["dtype"] else x
    _say(f"[case] naive random configuration {c}")
    check_case(tahq, xin, c["B"], c["S"], c["Cc"], c["dtype"], c["bits"], c["scale"])
