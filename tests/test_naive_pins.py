"""Pins of the backward-pass compressor's oracle (oracle/naive_oracle.c): Q_Naive of Alg. 1 steps 6-7 and
the appendix's gradient scaling g_hat = Q(c g)/c.  The paper fixes no formula, so the pins are what the
chosen reading (b-bit two's-complement fixed point with step 1/c) and the mathematics fix: explicit
rounding and clamping cases, the float64 definition, exactness on the grid, the half-step error bound,
exact invariance under power-of-two pre-scaling, the byte layout parsed independently.  CPU only."""
import math

import numpy as np
import pytest

import workloads
from oracle import n32, n64

ALL_BITS = tuple(range(2, 17))


def _gradient_like(batch, seq, scale=1.0, dtype_bits=False):
    """Config-5-like tensor (sparse spikes, all-zero tokens), optionally shrunk by a power of two."""
    w, x = workloads.generate(5, batch=batch, seq=seq)
    f = workloads.bf16_bits_to_f32(x) * np.float32(scale)
    return w, (workloads.f32_to_bf16_bits(f) if dtype_bits else np.ascontiguousarray(f, np.float32))


def test_round_half_to_even_then_clamp_to_twos_complement_range():
    c, b = 1.0, 4                                   # codes -8 .. 7
    cases = {0.5: 0, 1.5: 2, 2.5: 2, -0.5: 0, -1.5: -2, -2.5: -2, 0.49999997: 0, 6.5: 6, 7.4: 7, 7.5: 7, 8.0: 7,
             1e9: 7, -7.5: -8, -8.5: -8, -9.0: -8, -1e30: -8, float("inf"): 7, float("-inf"): -8, 0.0: 0, -0.0: 0}
    for g, q in cases.items():
        assert n32.code(g, c, b) == q, g
    assert n32.code(float("nan"), c, b) == -8       # a NaN product takes the lower bound
    # the bounds for every width
    for bits in ALL_BITS:
        lo, hi = -(2 ** (bits - 1)), 2 ** (bits - 1) - 1
        assert n32.code(1e20, 1.0, bits) == hi and n32.code(-1e20, 1.0, bits) == lo
        assert n32.code(hi + 0.5, 1.0, bits) == hi and n32.code(lo - 0.5, 1.0, bits) == lo
        assert n32.code(hi - 1.0, 1.0, bits) == hi - 1 and n32.code(lo + 1.0, 1.0, bits) == lo + 1


@pytest.mark.parametrize("bits", ALL_BITS)
def test_codes_match_the_float64_definition(bits):
    rng = np.random.default_rng(100 + bits)
    hi = 2 ** (bits - 1)
    g = (rng.standard_normal(4000) * hi * 0.6).astype(np.float32)
    g[:200] = (rng.integers(-hi - 2, hi + 2, size=200) + 0.5).astype(np.float32)      # exact ties, some out of range
    for c in (1.0, 0.25, 64.0):                     # powers of two: c*g is exact, float64 applies directly
        scaled = g / np.float32(c)
        got = np.array([n32.code(v, c, bits) for v in scaled])
        assert np.array_equal(got, n64.codes(scaled.astype(np.float64) * c, bits))
    for c in (3.0, 0.1, 1234.567):                  # otherwise the product is rounded to fp32 first (NumPy's multiply)
        scaled = (g / np.float32(c)).astype(np.float32)
        prod = (np.float32(c) * scaled).astype(np.float32)
        got = np.array([n32.code(v, c, bits) for v in scaled])
        assert np.array_equal(got, n64.codes(prod, bits))


@pytest.mark.parametrize("bits", (2, 4, 6, 7, 8, 10, 16))
def test_grid_values_are_exact_and_the_rest_is_within_half_a_step(bits):
    lo, hi = n64.code_range(bits)
    for c in (1.0, 2.0 ** 17, 2.0 ** -3):
        q = np.arange(lo, hi + 1) if bits <= 10 else np.linspace(lo, hi, 1500).astype(np.int64)
        for qi in q:
            g = np.float32(qi / c)
            assert n32.code(g, c, bits) == qi
            assert n32.value(int(qi), c) == g
    rng = np.random.default_rng(7)
    for c in (1.0, 2.0 ** 17, 1000.0, 0.3):
        g = rng.uniform(lo / c, hi / c, size=3000).astype(np.float32)
        back = np.array([n32.value(n32.code(v, c, bits), c) for v in g], np.float64)
        # half a step, plus the fp32 roundings of c*g and of q*(1/c) when c is not a power of two
        assert np.max(np.abs(back - g.astype(np.float64))) <= 0.5 / c + 4 * 2.0 ** -24 * np.abs(g).max()
    # beyond the range the value saturates
    assert n32.value(n32.code(1e30, 8.0, bits), 8.0) == hi / 8.0
    assert n32.value(n32.code(-1e30, 8.0, bits), 8.0) == lo / 8.0


def test_value_is_code_times_the_rounded_reciprocal():
    rng = np.random.default_rng(8)
    q = rng.integers(-32768, 32768, size=2000)
    for c in (1.0, 4096.0, 3.0, 0.1, 1e5, 7e-4):
        got = np.array([n32.value(int(v), c) for v in q], np.float32)
        assert np.array_equal(got.view(np.uint32), n64.values(q, c).view(np.uint32))
        if math.log2(c).is_integer():               # then "/ c" is exact
            assert np.array_equal(got, (q / c).astype(np.float32))


@pytest.mark.parametrize("dtype_name", ("f32", "bf16"))
@pytest.mark.parametrize("bits", (4, 6, 7, 8, 10, 13))
def test_stream_layout_parsed_independently(dtype_name, bits):
    bf16 = dtype_name == "bf16"
    w, x = _gradient_like(2, 5, dtype_bits=bf16)
    c = 2.0 ** 13
    cfg = n32.make_cfg(2, 5, w.hidden, n32.BF16 if bf16 else n32.F32, bits, c)
    packed = n32.encode(cfg, x)
    n = x.size
    assert packed.size == n32.packed_size(cfg) == 64 + n * bits // 8
    hdr, q = n64.parse_stream(packed, n, bits)
    assert bytes(packed[:4]) == b"TAHN"
    assert list(hdr[1:7]) == [1, int(bf16), 2, 5, w.hidden, bits]
    assert hdr[7:8].view("<f4")[0] == np.float32(c) and not hdr[8:].any()
    xf = (workloads.bf16_bits_to_f32(x) if bf16 else x).astype(np.float64).reshape(-1)
    assert np.array_equal(q, n64.codes(xf * c, bits))          # power-of-two c: the float64 product is exact
    lo, hi = n64.code_range(bits)
    assert q.min() >= lo and q.max() <= hi and (q < 0).any() and (q > 0).any()
    # decode, both output types, against the independent parse
    out = n32.decode(cfg, packed, n32.F32)
    assert np.array_equal(out.view(np.uint32), n64.values(q, c).view(np.uint32))
    out16 = n32.decode(cfg, packed, n32.BF16)
    assert np.array_equal(out16, workloads.f32_to_bf16_bits(n64.values(q, c)))


def test_negative_codes_are_twos_complement_fields():
    # -1 is the all-ones field, the lower bound is the field 100..0; element i sits at bits [b*i, b*i+b)
    for bits in (3, 6, 8, 10):
        lo, hi = n64.code_range(bits)
        x = np.zeros((1, 1, 32), np.float32)
        x[0, 0, 0], x[0, 0, 1], x[0, 0, 2], x[0, 0, 31] = -1.0, lo, hi, 1.0
        packed = n32.encode(n32.make_cfg(1, 1, 32, n32.F32, bits, 1.0), x)
        stream_bits = np.unpackbits(packed[64:], bitorder="little")
        assert stream_bits[:bits].all()
        assert list(stream_bits[bits:2 * bits]) == [0] * (bits - 1) + [1]
        assert list(stream_bits[2 * bits:3 * bits]) == [1] * (bits - 1) + [0]
        assert list(stream_bits[31 * bits:32 * bits]) == [1] + [0] * (bits - 1)
        assert stream_bits.sum() == bits + 1 + (bits - 1) + 1


@pytest.mark.parametrize("bits", (4, 8, 10))
def test_power_of_two_pre_scaling_is_exactly_scaling_the_tensor(bits):
    # g_hat = Q(c g)/c: with c = 2^k the codes are those of the tensor multiplied by 2^k under c = 1, and the
    # decoded values are those divided by 2^k, bit for bit
    w, x = _gradient_like(1, 6, scale=2.0 ** -7)
    k = 20
    a = n32.encode(n32.make_cfg(1, 6, w.hidden, n32.F32, bits, 2.0 ** k), x)
    b = n32.encode(n32.make_cfg(1, 6, w.hidden, n32.F32, bits, 1.0), x * np.float32(2.0 ** k))
    assert np.array_equal(a[64:], b[64:])
    da = n32.decode(n32.make_cfg(1, 6, w.hidden, n32.F32, bits, 2.0 ** k), a)
    db = n32.decode(n32.make_cfg(1, 6, w.hidden, n32.F32, bits, 1.0), b)
    assert np.array_equal(da, db * np.float32(2.0 ** -k))


def test_small_gradients_vanish_without_scaling_and_survive_with_it():
    # the appendix's motivation: magnitudes around 1e-5 underflow a fixed-point grid unless rescaled
    rng = np.random.default_rng(3)
    g = (rng.standard_normal((1, 4, 256)) * 1e-5).astype(np.float32)
    plain = n32.make_cfg(1, 4, 256, n32.F32, 8, 1.0)
    assert not n32.decode(plain, n32.encode(plain, g)).any()
    c = 2.0 ** 21                                     # 3 sigma -> about 63 of 127 codes
    scaled = n32.make_cfg(1, 4, 256, n32.F32, 8, c)
    back = n32.decode(scaled, n32.encode(scaled, g)).reshape(g.shape)
    assert np.max(np.abs(back - g)) <= 0.5 / c
    rel = np.linalg.norm(back - g) / np.linalg.norm(g)
    assert rel < 0.02
    # two more bits, a quarter of the error: the appendix's 8 -> 10 bit remedy at the same range
    fine = n32.make_cfg(1, 4, 256, n32.F32, 10, 4 * c)
    back10 = n32.decode(fine, n32.encode(fine, g)).reshape(g.shape)
    assert np.linalg.norm(back10 - g) < 0.3 * np.linalg.norm(back - g)


def test_encoding_a_decoded_tensor_reproduces_the_stream():
    w, x = _gradient_like(2, 3)
    for bits, c in ((6, 2.0 ** 12), (8, 2.0 ** 14), (10, 1000.0)):
        cfg = n32.make_cfg(2, 3, w.hidden, n32.F32, bits, c)
        first = n32.encode(cfg, x)
        again = n32.encode(cfg, n32.decode(cfg, first))
        assert np.array_equal(first, again)


def test_invalid_configurations_have_size_zero():
    ok = dict(batch=2, seq=3, hidden=64, dtype=0, bits=8, scale=1.0)
    assert n32.packed_size(n32.make_cfg(**ok)) == 64 + 2 * 3 * 64
    for kw in (dict(batch=0), dict(seq=0), dict(hidden=0), dict(hidden=48), dict(dtype=2), dict(bits=1), dict(bits=17),
               dict(scale=0.0), dict(scale=-1.0), dict(scale=float("nan")), dict(scale=float("inf"))):
        bad = dict(ok); bad.update(kw)
        assert n32.packed_size(n32.make_cfg(**bad)) == 0, kw
