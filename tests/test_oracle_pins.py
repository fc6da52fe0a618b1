"""Pins for the CPU oracle: every part is checked against something other than itself.

Closed forms, invariants, dense-matrix definitions, brute force on tiny inputs,
numpy's float16, a textbook min-max quantizer and an independent float64 decoder
of the byte stream.  Citations are to the paper's sections and equations.
"""
import itertools
import math

import numpy as np
import pytest
from scipy.linalg import hadamard

import workloads
from oracle import o32, o64

GS = (8, 16, 32, 64, 128)


# ---------------------------------------------------------------- Hadamard

@pytest.mark.parametrize("G", GS)
def test_butterfly_is_dense_sylvester_product(G):
    # Related work / Eq. 4: H_G in {+-1}^{GxG}; the butterfly must equal v @ H_G.
    rng = np.random.default_rng(G)
    Hm = hadamard(G).astype(np.float64)
    for _ in range(20):
        v = rng.standard_normal(G).astype(np.float32)
        got = o32.butterfly(v).astype(np.float64)
        want = v.astype(np.float64) @ Hm
        assert np.allclose(got, want, rtol=0, atol=2e-5 * np.abs(v).sum())


@pytest.mark.parametrize("G", GS)
def test_butterfly_rows_are_orthogonal_HHt_equals_G_I(G):
    # H_G H_G^T = G I_G, in exact integers: the butterfly of unit vectors gives the rows of H.
    rows = np.stack([o32.butterfly(np.eye(G, dtype=np.float32)[i]) for i in range(G)])
    assert set(np.unique(rows)) == {-1.0, 1.0}
    assert np.array_equal(rows, hadamard(G).astype(np.float32))
    assert np.array_equal(rows.astype(np.int64) @ rows.astype(np.int64).T, G * np.eye(G, dtype=np.int64))


@pytest.mark.parametrize("G", GS)
def test_butterfly_twice_is_G_times_identity_exactly_on_small_integers(G):
    rng = np.random.default_rng(7)
    v = rng.integers(-1024, 1025, size=G).astype(np.float32)
    assert np.array_equal(o32.butterfly(o32.butterfly(v)), G * v)


@pytest.mark.parametrize("G", GS)
def test_forward_transform_matches_dense_definition_and_preserves_norm(G):
    # Eq. 4: alpha P_d (1/sqrt G) H_G with dense matrices in float64.
    rng = np.random.default_rng(11 + G)
    for d in (0, 1, 5, G - 1):
        v = rng.standard_normal(G).astype(np.float32)
        got = o32.forward_transform(v, d).astype(np.float64)
        want = o64.forward_transform(v, d)
        assert np.allclose(got, want, rtol=0, atol=1e-5)
        assert math.isclose(np.linalg.norm(got), np.linalg.norm(v.astype(np.float64)), rel_tol=1e-5)


@pytest.mark.parametrize("G", GS)
def test_inverse_transform_inverts(G):
    rng = np.random.default_rng(3)
    for d in (0, 2, G - 1):
        v = rng.standard_normal(G).astype(np.float32)
        back = o32.inverse_transform(o32.forward_transform(v, d), d)
        assert np.allclose(back, v, rtol=0, atol=1e-5)
        # dense definition of the inverse (apply H^T, then P_d)
        y = o32.forward_transform(v, d)
        assert np.allclose(o32.inverse_transform(y, d), o64.inverse_transform(y, d), rtol=0, atol=1e-5)


def test_inverse_transform_exact_on_power_of_two_scaled_integers():
    # G = 64: 1/sqrt(G) = 1/8 is exact, so integer tiles round-trip bit for bit.
    rng = np.random.default_rng(5)
    v = (rng.integers(-512, 513, size=64) * 8).astype(np.float32)
    for d in (0, 9, 63):
        assert np.array_equal(o32.inverse_transform(o32.forward_transform(v, d), d), v)


@pytest.mark.parametrize("G", GS)
def test_pivot_swap_is_a_permutation_and_an_involution(G):
    # P_d swaps coordinates 1 and d.  Isolate it: with H removed (apply the butterfly again and
    # divide by G) what is left of the forward transform is the swap.
    v = np.arange(1, G + 1, dtype=np.float32) * 8
    for d in (0, 1, G // 3, G - 1):
        y = o32.butterfly(v.copy())                      # H v
        t = v.copy(); t[[0, d]] = t[[d, 0]]
        assert np.array_equal(o32.butterfly(t), o32.butterfly(v @ o64.swap_matrix(G, d).astype(np.float32)))
        assert sorted(t) == sorted(v)
        t2 = t.copy(); t2[[0, d]] = t2[[d, 0]]
        assert np.array_equal(t2, v)
        # after the swap the pivot leads, so every transformed entry carries +-pivot/sqrt(G)
        w = np.zeros(G, np.float32); w[d] = 16.0
        assert np.allclose(o32.forward_transform(w, d), 16.0 / math.sqrt(G), rtol=1e-6)
        del y


# ------------------------------------------------------------------ log

def test_log_polynomial_accuracy():
    u = np.concatenate([np.geomspace(1e-9, 2.0, 20001), np.linspace(0.4, 1.1, 5001), [1.0, 0.5, 0.25, 1e-8]])
    u = u.astype(np.float32)
    got = np.array([o32.log(x) for x in u], np.float64)
    assert np.max(np.abs(got - np.log(u.astype(np.float64)))) <= 1.1e-5


def test_log_is_monotone_enough_for_ranking():
    u = np.geomspace(1e-8, 1.0, 4001).astype(np.float32)
    got = np.array([o32.log(x) for x in u])
    # never decreasing by more than the stated error
    assert np.all(np.diff(got) > -2.2e-5)


# -------------------------------------------------------------- entropy

@pytest.mark.parametrize("G", GS)
def test_entropy_closed_forms(G):
    # Sec. 3.2: H is high for evenly spread energy (ln G) and low for a sharp outlier (0):
    # this fixes the sign that Eq. 2 prints without a minus.
    tol = 3e-5
    assert abs(o32.entropy(np.full(G, 2.5, np.float32)) - math.log(G)) < tol
    assert abs(o32.entropy(np.full(G, -1e-3, np.float32)) - math.log(G)) < tol
    onehot = np.zeros(G, np.float32); onehot[G // 2] = -7.0
    assert abs(o32.entropy(onehot)) < tol
    assert o32.entropy(np.zeros(G, np.float32)) == 0.0
    for m in (2, 4, 8, min(16, G)):
        v = np.zeros(G, np.float32); v[:m] = 3.0; v[1] = -3.0
        assert abs(o32.entropy(v) - math.log(m)) < tol


@pytest.mark.parametrize("G", GS)
def test_entropy_matches_float64_definition_bounds_and_scale_invariance(G):
    rng = np.random.default_rng(G + 1)
    tiles = rng.standard_normal((200, G)).astype(np.float32)
    tiles[::7, 3] *= 50
    tiles[::11] = rng.uniform(-8, 8, size=(len(tiles[::11]), G)).astype(np.float32)
    want = o64.entropy(tiles)
    got = np.array([o32.entropy(t) for t in tiles])
    assert np.max(np.abs(got - want)) < 3e-5
    assert np.all(got > -3e-5) and np.all(got < math.log(G) + 3e-5)
    scaled = np.array([o32.entropy(t * np.float32(37.0)) for t in tiles])
    assert np.max(np.abs(scaled - got)) < 3e-5


def test_entropy_monotone_under_spreading():
    # moving mass from the peak to an empty slot raises H
    G = 64
    v = np.zeros(G, np.float32); v[0] = 64.0
    last = o32.entropy(v)
    for k in range(1, G):
        v[0] -= 1.0; v[k] = 1.0
        h = o32.entropy(v)
        assert h > last - 1e-5
        last = h


def test_tile_stats_entropy_equals_per_tile_function_and_bf16_widening():
    w, x = workloads.generate(5, batch=1, seq=8)
    cfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, o32.BF16, w.budget_bits)
    H, pivot, mn, mx = o32.tile_stats(cfg, x)
    xf = workloads.bf16_bits_to_f32(x).reshape(-1, w.tile)
    for j in range(0, len(H), 97):
        assert H[j] == np.float32(o32.entropy(xf[j]))
    assert np.max(np.abs(H - o64.entropy(xf))) < 3e-5


# --------------------------------------------------------- outlier test

def test_outlier_heuristic_eq3():
    G = 64
    rng = np.random.default_rng(0)
    tiles = rng.standard_normal((500, G)).astype(np.float32)
    tiles[::5, 17] = 30.0
    flag64, d64 = o64.outlier(tiles)
    for t, f, d in zip(tiles, flag64, d64):
        got_f, got_d = o32.outlier(t)
        assert got_d == d
        a = np.sort(np.abs(t.astype(np.float64)))
        r = a[-1] / (a[-2] + 1e-8)
        if abs(r - 2.0) > 1e-4:
            assert got_f == f == (r > 2.0)


def test_outlier_ties_and_special_taus():
    G = 32
    v = np.zeros(G, np.float32); v[4] = -9.0; v[20] = 9.0; v[7] = 1.0
    flag, d = o32.outlier(v)
    assert d == 4 and not flag                       # two equal maxima: r ~ 1, lowest index wins
    v[20] = 1.0
    assert o32.outlier(v) == (True, 4)
    rng = np.random.default_rng(1)
    for _ in range(50):
        t = rng.standard_normal(G).astype(np.float32)
        assert o32.outlier(t, tau=0.0)[0] is True        # tau = 0: always transform (App. tau study)
        assert o32.outlier(t, tau=float("inf"))[0] is False
        big = t.copy(); big[3] = 1e6
        assert o32.outlier(big, tau=float("inf"))[0] is False
    assert o32.outlier(np.zeros(G, np.float32), tau=0.0) == (False, 0)
    assert o32.outlier(np.zeros(G, np.float32), tau=2.0) == (False, 0)


# ------------------------------------------------------------ float16

def test_fp16_conversions_against_numpy_float16():
    rng = np.random.default_rng(2)
    xs = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 5, 4000).astype(np.float32),
        np.array([0.0, 65504.0, -65504.0, 65519.0, 65520.0, -1e9, 1e9, 6e-8, 5.96e-8, 2.98e-8, 2.981e-8,
                  1e-10, -1e-10, 6.1e-5, 6.09e-5, 1.0, 1.00048828125, 1.0009765625], np.float32),
        np.arange(0, 2048, dtype=np.float32) / np.float32(1024.0),
    ]).astype(np.float32)
    with np.errstate(over="ignore"):
        rne_np = xs.astype(np.float16)
    for x, h_np in zip(xs, rne_np):
        h = o32.fp16_rne(x)
        assert h == int(h_np.view(np.uint16)), (x, h, h_np)
    all16 = np.arange(0, 0x7c00, dtype=np.uint16)
    for h in list(all16[::37]) + [0x0001, 0x03ff, 0x0400, 0x7bff, 0x8001, 0xfbff]:
        assert o32.fp16_widen(int(h)) == float(np.uint16(h).view(np.float16))


@pytest.mark.filterwarnings("ignore:overflow encountered")
def test_fp16_directed_rounding_brackets_the_value():
    rng = np.random.default_rng(3)
    xs = rng.standard_normal(3000).astype(np.float32) * np.float32(10.0) ** rng.integers(-10, 5, 3000).astype(np.float32)
    xs = np.concatenate([xs, np.array([0.0, 1.0, -1.0, 3e-8, -3e-8, 1e-12, -1e-12, 65504.0, -65504.0], np.float32)])
    for x in xs:
        lo = np.uint16(o32.fp16_down(x)).view(np.float16)
        hi = np.uint16(o32.fp16_up(x)).view(np.float16)
        assert float(lo) <= float(x) <= float(hi)
        # tight: one float16 step further would cross x
        assert float(np.nextafter(lo, np.float16(np.inf))) > float(x)
        assert float(np.nextafter(hi, np.float16(-np.inf))) < float(x)
        assert o32.fp16_down(x) != 0x8000 and o32.fp16_up(x) != 0x8000
    # saturation beyond the float16 range
    assert np.uint16(o32.fp16_down(-1e9)).view(np.float16) == np.float16(-65504)
    assert np.uint16(o32.fp16_up(1e9)).view(np.float16) == np.float16(65504)
    assert np.uint16(o32.fp16_down(1e9)).view(np.float16) == np.float16(65504)


def test_bf16_rne_against_torch():
    import torch
    rng = np.random.default_rng(4)
    xs = (rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000)).astype(np.float32)
    xs = np.concatenate([xs, np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.3895314e38], np.float32)])
    want = torch.from_numpy(xs).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([o32.bf16_rne(x) for x in xs], np.uint16)
    assert np.array_equal(got, want)
    assert np.array_equal(workloads.f32_to_bf16_bits(xs), want)


# ---------------------------------------------------------- quantizer

@pytest.mark.parametrize("b", (2, 3, 4))
def test_quantizer_half_step_bound_and_coverage(b):
    rng = np.random.default_rng(10 + b)
    L = (1 << b) - 1
    for scale in (1e-3, 1.0, 40.0, 3e3):
        for _ in range(40):
            y = (rng.standard_normal(64) * scale).astype(np.float32)
            mn, mx = float(y.min()), float(y.max())
            s16, z16 = o32.quant_params(mn, mx, b)
            sf, mnf = o32.fp16_widen(s16), o32.fp16_widen(z16)
            assert mnf <= mn and mnf + L * sf >= mx          # outward-rounded metadata covers the range
            for v in y:
                q = o32.quant_code(v, s16, z16, b)
                assert 0 <= q <= L
                err = abs(o32.dequant(q, s16, z16) - float(v))
                assert err <= sf / 2 * (1 + 2.0 ** -10) + 1e-12


def test_quantizer_rounds_half_to_even_and_clamps():
    s16 = o32.fp16_rne(1.0); z16 = o32.fp16_rne(0.0)
    assert [o32.quant_code(v, s16, z16, 4) for v in (0.5, 1.5, 2.5, 3.5, 14.5, 15.4, 99.0, -3.0)] == \
        [0, 2, 2, 4, 14, 15, 15, 0]
    assert [o32.quant_code(v, s16, z16, 3) for v in (6.5, 7.49, 7.5, 8.0)] == [6, 7, 7, 7]
    assert [o32.quant_code(v, s16, z16, 2) for v in (0.5, 1.5, 2.5, 2.51, 3.5, 9.0, -1.0)] == [0, 2, 2, 3, 3, 3, 0]
    assert o32.quant_code(float("nan"), s16, z16, 4) == 0


def test_constant_and_zero_tiles_have_unit_scale_and_zero_codes():
    for c in (0.0, 3.25, -0.5):
        s16, z16 = o32.quant_params(c, c, 3)
        zf = o32.fp16_widen(z16)
        if zf == c:
            assert s16 == 0x3c00
        assert o32.quant_code(c, s16, z16, 3) == 0 or o32.fp16_widen(s16) < 1.0


def test_quantizer_agrees_with_textbook_minmax_when_metadata_is_exact():
    # Values on a binary grid with float16-exact min and scale: codes must equal the float64
    # textbook min-max group quantizer, except exactly-half ties which both round to even.
    rng = np.random.default_rng(21)
    for b in (2, 3, 4):
        L = (1 << b) - 1
        for _ in range(50):
            q_true = rng.integers(0, L + 1, size=64)
            q_true[:2] = (0, L)
            frac = rng.uniform(-0.45, 0.45, size=64); frac[:2] = 0
            frac = np.clip(q_true + frac, 0, L) - q_true          # keep min and max at codes 0 and L
            mn, s = -2.0, 0.25
            y = (mn + (q_true + frac) * s).astype(np.float32)
            s16, z16 = o32.quant_params(float(y.min()), float(y.max()), b)
            assert o32.fp16_widen(s16) == s and o32.fp16_widen(z16) == mn
            got = np.array([o32.quant_code(v, s16, z16, b) for v in y])
            want, s64, mn64 = o64.minmax_group_quantize(y[None, :], b)
            assert np.array_equal(got, want[0].astype(np.int64))
            assert np.array_equal(got, q_true)


# ---------------------------------------------------------- allocation

def test_allocation_brute_force_top_k_maximises_total_entropy():
    rng = np.random.default_rng(8)
    # tiny tensors: hidden = 2 tiles of 32, seq chosen so n <= 12
    for n_tok, budget in ((3, 3.5), (4, 3.25), (6, 3.5), (5, 3.4), (6, 3.0), (6, 4.0)):
        cfg = o32.make_cfg(1, n_tok, 64, 32, o32.F32, budget)
        n = n_tok * 2
        H = rng.standard_normal(n).astype(np.float32)
        k = o32.k_per_unit(cfg)
        assert k == o64.k_per_unit(n, budget)
        width = o32.allocate(cfg, H)
        assert (width == 4).sum() == k and set(np.unique(width)) <= {3, 4}
        best = max(itertools.combinations(range(n), k), key=lambda s: H[list(s)].astype(np.float64).sum()) if k else ()
        assert set(np.nonzero(width == 4)[0]) == set(best)
        assert math.isclose(width.mean(), 3 + k / n)


def test_allocation_ties_go_to_lower_index_and_per_sample():
    cfg = o32.make_cfg(2, 4, 64, 32, o32.F32, 3.5)      # 2 samples x 8 tiles, k = 4 each
    H = np.array([1, 1, 1, 1, 1, 1, 1, 1, 0, 5, 5, 0, 5, 5, 5, 0], np.float32)
    width = o32.allocate(cfg, H)
    assert list(width[:8]) == [4, 4, 4, 4, 3, 3, 3, 3]
    assert list(width[8:]) == [3, 4, 4, 3, 4, 4, 3, 3]
    assert np.array_equal(width, o64.allocate(H, 2, 4))
    # whole-tensor ranking (scope 1): k = 8 of 16
    cfg1 = o32.make_cfg(2, 4, 64, 32, o32.F32, 3.5, scope=1)
    w1 = o32.allocate(cfg1, H)
    assert list(w1) == [4, 4, 4, 3, 3, 3, 3, 3, 3, 4, 4, 3, 4, 4, 4, 3]


def test_mean_bit_width_equals_budget_on_all_five_configs():
    for w in workloads.CONFIGS:
        cfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
        n = w.seq * (w.hidden // w.tile)
        k = o32.k_per_unit(cfg)
        assert 3 + k / n == w.budget_bits


def test_allocation_matches_lexsort_on_random_entropies_with_duplicates():
    rng = np.random.default_rng(9)
    cfg = o32.make_cfg(3, 50, 256, 32, o32.F32, 3.3)
    T = o32.n_tiles(cfg)
    H = rng.integers(0, 40, size=T).astype(np.float32) / np.float32(8)     # many duplicates
    assert np.array_equal(o32.allocate(cfg, H), o64.allocate(H, 3, o32.k_per_unit(cfg)))


# ------------------------------------- allocation tiles larger than G

@pytest.mark.parametrize("G,m", [(32, 2), (64, 3), (64, 16), (128, 64)])
def test_allocation_tile_entropy_closed_forms_and_float64_definition(G, m):
    # Sec. 3.2, Eq. 1-2 on A = m*G channels: uniform magnitudes -> ln A; one-hot -> 0; j equal entries -> ln j.
    A = G * m
    tol = 3e-5 * max(1.0, math.log(A))
    assert abs(o32.entropy_alloc(np.full(A, -0.75, np.float32), G) - math.log(A)) < tol
    onehot = np.zeros(A, np.float32); onehot[A - 3] = 9.0
    assert abs(o32.entropy_alloc(onehot, G)) < tol
    assert o32.entropy_alloc(np.zeros(A, np.float32), G) == 0.0
    for j in (2, G, G + 1, A // 2):
        v = np.zeros(A, np.float32); v[np.linspace(0, A - 1, j).astype(int)] = 3.0
        assert abs(o32.entropy_alloc(v, G) - math.log(j)) < tol
    rng = np.random.default_rng(31)
    v = rng.standard_normal((20, A)).astype(np.float32) * np.exp(rng.standard_normal((20, A))).astype(np.float32)
    want = o64.entropy(v)
    got = np.array([o32.entropy_alloc(t, G) for t in v])
    assert np.max(np.abs(got - want)) < tol
    # the split into quantization tiles only fixes the rounding order
    if A <= 128:
        assert np.max(np.abs(got - np.array([o32.entropy(t) for t in v]))) < tol


def test_allocation_tile_of_one_quantization_tile_is_the_default():
    rng = np.random.default_rng(32)
    for G in GS:
        for t in rng.standard_normal((50, G)).astype(np.float32):
            assert o32.entropy_alloc(t, G) == o32.entropy(t)
    w, x = workloads.generate(2, batch=2, seq=24)
    a = o32.encode(o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.4), x)
    b = o32.encode(o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.4, alloc_tile=w.tile), x)
    assert np.array_equal(a, b)
    assert a[:64].view("<u4")[14] == w.tile


@pytest.mark.parametrize("index,shape,m", [(1, dict(batch=2, seq=12), 2), (2, dict(batch=2, seq=24), 4),
                                           (4, dict(batch=2, seq=10), 8), (5, dict(batch=1, seq=16), 5)])
def test_allocation_over_tiles_of_several_quantization_tiles(index, shape, m):
    w, x = workloads.generate(index, **shape)
    G, A = w.tile, w.tile * m
    assert w.hidden % A == 0
    cfg = o32.make_cfg(w.batch, w.seq, w.hidden, G, w.dtype, 3.3, alloc_tile=A)
    T = o32.n_tiles(cfg)
    nA = w.seq * (w.hidden // A)
    kA = o32.k_per_unit(cfg)
    assert kA == o64.k_per_unit(nA, 3.3)
    packed = o32.encode(cfg, x)
    assert packed.size == o32.packed_size(cfg) == o64.section_offsets(T, G, w.batch, kA * m)["total"]
    out64, s = o64.decode_stream(packed, T, G, w.batch, kA * m)
    hdr = s["header"].view("<u4")
    assert list(hdr[1:9]) == [1, w.dtype, w.batch, w.seq, w.hidden, G, 0, kA] and hdr[14] == A
    # entropies of the allocation tiles against the float64 definition on A channels
    xf = (x if w.dtype == workloads.F32 else workloads.bf16_bits_to_f32(x)).astype(np.float64)
    HA = o32.alloc_entropies(cfg, x)
    assert HA.shape == (w.batch * nA,)
    assert np.max(np.abs(HA - o64.entropy(xf.reshape(-1, A)))) < 5e-5
    # one width per allocation tile: the top kA of each sample, shared by its m quantization tiles
    wantA = o64.allocate(HA, w.batch, kA)
    assert np.array_equal(s["width"], np.repeat(wantA, m))
    assert np.array_equal(o32.allocate(cfg, HA), np.repeat(wantA, m))
    assert np.array_equal(s["ranks"], s["rank_of"][::64])
    # quantization is untouched by A: pivots and ranges are those of the quantization tiles
    _, pivot, mn, mx = o32.tile_stats(cfg, x)
    assert np.array_equal(s["pivot"], pivot)
    sf = s["scale"].astype(np.float64); zf = s["zero"].astype(np.float64)
    L = (1 << s["width"]) - 1
    assert np.all(zf <= mn) and np.all(zf + L * sf >= mx) and np.all(s["codes"] <= L[:, None])
    out32 = o32.decode(cfg, packed, o32.F32).reshape(T, G).astype(np.float64)
    scale = np.maximum(np.abs(out64).max(axis=1, keepdims=True), 1e-30)
    assert np.max(np.abs(out32 - out64) / scale) < 1e-5
    err = np.linalg.norm(out64 - xf.reshape(T, G), axis=1)
    assert np.all(err <= sf / 2 * math.sqrt(G) * (1 + 1e-3) + 1e-6 * np.abs(xf.reshape(T, G)).max(axis=1))


def test_token_level_allocation_is_the_special_case_A_equals_C():
    # Sec. 3.2: with A = C every allocation tile is a whole token, so a token's tiles share one width and
    # the INT4 tokens are the top-p% of the per-token entropies.
    w, x = workloads.generate(2, batch=2, seq=40)
    G, Cc = w.tile, w.hidden
    cfg = o32.make_cfg(w.batch, w.seq, Cc, G, w.dtype, 3.25, alloc_tile=Cc)
    assert o32.k_per_unit(cfg) == 10
    s = o64.parse_stream(o32.encode(cfg, x), o32.n_tiles(cfg), G, w.batch, 10 * (Cc // G))
    per_token = s["width"].reshape(w.batch, w.seq, Cc // G)
    assert np.all(per_token == per_token[:, :, :1])
    xf = (x if w.dtype == workloads.F32 else workloads.bf16_bits_to_f32(x)).astype(np.float64)
    Htok = o64.entropy(xf.reshape(-1, Cc)).reshape(w.batch, w.seq)
    for i in range(w.batch):
        chosen = set(np.nonzero(per_token[i, :, 0] == 4)[0])
        order = np.argsort(-Htok[i], kind="stable")
        # float64 ranking agrees wherever the gap at the cut is above the fp32 evaluation error
        sure_in = {int(t) for t in order[:10] if Htok[i, t] - Htok[i, order[10]] > 1e-4}
        sure_out = {int(t) for t in order[10:] if Htok[i, order[9]] - Htok[i, t] > 1e-4}
        assert len(chosen) == 10 and sure_in <= chosen and not (sure_out & chosen)


def test_allocation_tile_must_align_with_quantization_tiles_and_divide_the_hidden_size():
    assert o32.packed_size(o32.make_cfg(1, 4, 384, 64, o32.F32, 3.5, alloc_tile=96)) == 0     # not a multiple of G
    assert o32.packed_size(o32.make_cfg(1, 4, 384, 64, o32.F32, 3.5, alloc_tile=256)) == 0    # does not divide C
    assert o32.packed_size(o32.make_cfg(1, 4, 384, 64, o32.F32, 3.5, alloc_tile=32)) == 0     # below G
    assert o32.packed_size(o32.make_cfg(1, 4, 384, 64, o32.F32, 3.5, alloc_tile=192)) > 0


# ------------------- tiles of 8 and 16 channels, hidden sizes that are not powers of two

@pytest.mark.parametrize("G,C_,dtype_name,low", [(8, 200, "f32", 3), (16, 208, "bf16", 3), (8, 64, "bf16", 2),
                                                 (16, 1600, "f32", 2), (64, 1600, "bf16", 3), (32, 1600, "f32", 3),
                                                 # any pair of neighbouring widths, 1/2 bits up to 7/8 bits
                                                 (8, 64, "f32", 1), (64, 640, "bf16", 1), (128, 256, "bf16", 4),
                                                 (32, 160, "bf16", 5), (16, 208, "f32", 6), (64, 1600, "f32", 7),
                                                 (8, 200, "bf16", 7)])
def test_small_tiles_and_hidden_1600_streams_parse_and_decode_in_float64(G, C_, dtype_name, low):
    # the tile-size ablation uses tiles of 8 channels; 1600 is a hidden size with 25 tiles of 64 per token
    rng = np.random.default_rng(G + C_)
    B, S = 2, 9
    x = rng.standard_normal((B, S, C_)).astype(np.float32)
    x[:, :, 5::37] *= 25.0
    x[1, 2, :] = 0.0
    dtype = o32.BF16 if dtype_name == "bf16" else o32.F32
    xin = workloads.f32_to_bf16_bits(x) if dtype else x
    budget = low + 0.3
    cfg = o32.make_cfg(B, S, C_, G, dtype, budget, low_bits=low)
    packed = o32.encode(cfg, xin)
    T = o32.n_tiles(cfg)
    k = o32.k_per_unit(cfg)
    assert k == o64.k_per_unit(S * (C_ // G), np.float32(budget), low=low)     # the budget is an fp32 field
    assert packed.size == o32.packed_size(cfg) == o64.section_offsets(T, G, B, k, low=low)["total"]
    out64, s = o64.decode_stream(packed, T, G, B, k, low=low)
    hdr = s["header"].view("<u4")
    assert list(hdr[1:9]) == [1, dtype, B, S, C_, G, 0, k] and hdr[14] == G and hdr[15] == low
    H, pivot, mn, mx = o32.tile_stats(cfg, xin)
    xf = (workloads.bf16_bits_to_f32(xin) if dtype else x).reshape(T, G).astype(np.float64)
    assert np.max(np.abs(H - o64.entropy(xf))) < 3e-5
    assert np.array_equal(s["width"], o64.allocate(H, B, k, low=low))
    assert np.array_equal(s["ranks"], s["rank_of"][::64])
    assert np.array_equal(s["pivot"], pivot)
    flag64, d64 = o64.outlier(xf)
    assert np.array_equal(pivot & 0x7F, np.where(flag64, d64, 0)) and np.array_equal(pivot >> 7, flag64.astype(np.uint8))
    sf = s["scale"].astype(np.float64); zf = s["zero"].astype(np.float64)
    L = (1 << s["width"]) - 1
    assert np.all(zf <= mn) and np.all(zf + L * sf >= mx) and np.all(s["codes"] <= L[:, None])
    out32 = o32.decode(cfg, packed, o32.F32).reshape(T, G).astype(np.float64)
    scale = np.maximum(np.abs(out64).max(axis=1, keepdims=True), 1e-30)
    assert np.max(np.abs(out32 - out64) / scale) < 1e-5
    err = np.linalg.norm(out64 - xf, axis=1)
    assert np.all(err <= sf / 2 * math.sqrt(G) * (1 + 1e-3) + 1e-6 * np.abs(xf).max(axis=1))


# ------------------------- a seeded sweep over combinations of the options

def _sweep_cases(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        G = int(rng.choice([8, 16, 32, 64, 128]))
        M = int(rng.choice([1, 2, 3, 4, 6, 10]))
        B, S = int(rng.choice([1, 2, 3])), int(rng.choice([1, 5, 23, 70]))
        low = int(rng.choice([3, 3, 2, 1, 4, 5, 6, 7]))
        divisors = [d for d in range(1, M + 1) if M % d == 0]
        m = int(rng.choice(divisors)) if rng.random() < 0.5 else 1
        out.append(dict(B=B, S=S, G=G, M=M, dtype=int(rng.integers(0, 2)), low=low, m=m, scope=int(rng.random() < 0.3),
                        budget=float(np.float32(low + rng.choice([0.0, 1.0, rng.uniform(0.05, 0.95)]))),
                        tau=float(rng.choice([2.0, 1.5, 5.0])), seed=int(rng.integers(0, 2 ** 31))))
    return out


@pytest.mark.parametrize("c", _sweep_cases(64, seed=77), ids=lambda c: "{B}x{S}x{M}tiles_g{G}_d{dtype}_lo{low}_m{m}_s{scope}".format(**c))
def test_option_combinations_parse_and_decode_independently_in_float64(c):
    # every combination of tile width, dtype, widths, allocation tile, scope and tau goes through the independent
    # float64 statement: size, header, allocation from the entropies, rank table, pivots, coverage, decode, error bound
    rng = np.random.default_rng(c["seed"])
    B, S, G, M, low, m = c["B"], c["S"], c["G"], c["M"], c["low"], c["m"]
    Cc = G * M
    x = rng.standard_normal((B, S, Cc)).astype(np.float32) * np.exp(rng.standard_normal((B, S, 1))).astype(np.float32)
    x[:, :, ::max(1, Cc // 5)] *= 25.0
    if S > 4:
        x[:, ::4, :] = 0.0
    xin = workloads.f32_to_bf16_bits(x) if c["dtype"] else x
    cfg = o32.make_cfg(B, S, Cc, G, c["dtype"], c["budget"], tau=c["tau"], scope=c["scope"], alloc_tile=G * m if m > 1 else 0,
                       low_bits=low)
    U = 1 if c["scope"] else B
    T = o32.n_tiles(cfg)
    kA = o32.k_per_unit(cfg)
    assert kA == o64.k_per_unit(T // m // U, np.float32(c["budget"]), low=low)
    packed = o32.encode(cfg, xin)
    assert packed.size == o32.packed_size(cfg) == o64.section_offsets(T, G, U, kA * m, low=low)["total"]
    out64, s = o64.decode_stream(packed, T, G, U, kA * m, low=low)
    hdr = s["header"].view("<u4")
    assert list(hdr[1:9]) == [1, c["dtype"], B, S, Cc, G, c["scope"], kA] and hdr[14] == G * m and hdr[15] == low
    xf = (workloads.bf16_bits_to_f32(xin) if c["dtype"] else x).astype(np.float64)
    HA = o32.alloc_entropies(cfg, xin)
    assert np.max(np.abs(HA - o64.entropy(xf.reshape(-1, G * m)))) < 5e-5
    assert np.array_equal(s["width"], np.repeat(o64.allocate(HA, U, kA, low=low), m))
    assert np.array_equal(s["ranks"], s["rank_of"][::64])
    flag64, d64 = o64.outlier(xf.reshape(T, G), tau=c["tau"])
    _, pivot, mn, mx = o32.tile_stats(cfg, xin)
    assert np.array_equal(s["pivot"], pivot)
    # float64 and fp32 agree on the outlier test except within rounding of the threshold
    a = np.sort(np.abs(xf.reshape(T, G)), axis=1)
    clear = np.abs(a[:, -1] - c["tau"] * (a[:, -2] + 1e-8)) > 1e-5 * np.maximum(a[:, -1], 1e-30)
    assert np.array_equal((pivot >> 7)[clear], flag64.astype(np.uint8)[clear])
    assert np.array_equal((pivot & 0x7F)[flag64 & clear], d64[flag64 & clear])
    sf = s["scale"].astype(np.float64); zf = s["zero"].astype(np.float64)
    L = (1 << s["width"]) - 1
    # the step is (max - zero)/L rounded to fp32 and then up to binary16: the coded range reaches the maximum up to
    # that one fp32 rounding (when the quotient is itself a binary16 value, rounding up adds no slack)
    assert np.all(zf <= mn) and np.all(zf + L * sf >= mx - 2.0 ** -22 * (mx - zf)) and np.all(s["codes"] <= L[:, None])
    out32 = o32.decode(cfg, packed, o32.F32).reshape(T, G).astype(np.float64)
    scale = np.maximum(np.abs(out64).max(axis=1, keepdims=True), 1e-30)
    assert np.max(np.abs(out32 - out64) / scale) < 1e-5
    err = np.linalg.norm(out64 - xf.reshape(T, G), axis=1)
    assert np.all(err <= sf / 2 * math.sqrt(G) * (1 + 1e-3) + 1e-6 * np.abs(xf.reshape(T, G)).max(axis=1))


# ------------------------------------------- the INT2/INT3 mix (lo = 2)

def test_low_bits_changes_the_two_widths_the_budget_range_and_the_count():
    # appendix on bit allocation: 80% INT2 + 20% INT3 is budget 2.2 with widths {2, 3}
    cfg = o32.make_cfg(2, 10, 512, 64, o32.F32, 2.2, low_bits=2)
    n = 10 * 8
    assert o32.k_per_unit(cfg) == 16 == o64.k_per_unit(n, 2.2, low=2)
    H = np.arange(2 * n, dtype=np.float32)
    width = o32.allocate(cfg, H)
    assert set(np.unique(width)) == {2, 3} and (width == 3).sum() == 32
    assert np.array_equal(width, o64.allocate(H, 2, 16, low=2))
    assert math.isclose(width.mean(), 2.2)
    # the budget must lie in [lo, lo + 1]
    assert o32.packed_size(o32.make_cfg(2, 10, 512, 64, o32.F32, 3.2, low_bits=2)) == 0
    assert o32.packed_size(o32.make_cfg(2, 10, 512, 64, o32.F32, 1.9, low_bits=2)) == 0
    assert o32.packed_size(o32.make_cfg(2, 10, 512, 64, o32.F32, 2.2, low_bits=3)) == 0
    assert o32.packed_size(o32.make_cfg(2, 10, 512, 64, o32.F32, 2.2, low_bits=4)) == 0
    assert o32.packed_size(o32.make_cfg(2, 10, 512, 64, o32.F32, 3.0, low_bits=2)) > 0
    # lo = 3 written out is the default
    w, x = workloads.generate(1, batch=1, seq=8)
    a = o32.encode(o32.make_cfg(1, 8, w.hidden, w.tile, w.dtype, 3.5), x)
    b = o32.encode(o32.make_cfg(1, 8, w.hidden, w.tile, w.dtype, 3.5, low_bits=3), x)
    assert np.array_equal(a, b) and a[:64].view("<u4")[15] == 3


@pytest.mark.parametrize("index,shape,budget", [(1, dict(batch=1, seq=16), 2.2), (2, dict(batch=2, seq=24), 2.5),
                                                (3, dict(batch=2, seq=8), 2.0), (4, dict(batch=2, seq=40), 2.2),
                                                (5, dict(batch=2, seq=16), 3.0), (4, dict(batch=1, seq=12), 2.75)])
def test_int2_int3_stream_parses_and_decodes_independently_in_float64(index, shape, budget):
    w, x = workloads.generate(index, **shape)
    cfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget, low_bits=2)
    packed = o32.encode(cfg, x)
    T, G = o32.n_tiles(cfg), w.tile
    k = o32.k_per_unit(cfg)
    assert packed.size == o32.packed_size(cfg) == o64.section_offsets(T, G, w.batch, k, low=2)["total"]
    out64, s = o64.decode_stream(packed, T, G, w.batch, k, low=2)
    hdr = s["header"].view("<u4")
    assert list(hdr[1:9]) == [1, w.dtype, w.batch, w.seq, w.hidden, G, 0, k] and hdr[15] == 2
    H, pivot, mn, mx = o32.tile_stats(cfg, x)
    assert np.array_equal(s["bits"].reshape(w.batch, -1).sum(axis=1), np.full(w.batch, k))
    assert np.array_equal(s["width"], o64.allocate(H, w.batch, k, low=2))
    assert np.array_equal(s["ranks"], s["rank_of"][::64])
    assert np.array_equal(s["pivot"], pivot)
    sf = s["scale"].astype(np.float64); zf = s["zero"].astype(np.float64)
    L = (1 << s["width"]) - 1
    assert set(np.unique(L)) <= {3, 7}
    assert np.all(zf <= mn) and np.all(zf + L * sf >= mx) and np.all(s["codes"] <= L[:, None])
    out32 = o32.decode(cfg, packed, o32.F32).reshape(T, G).astype(np.float64)
    scale = np.maximum(np.abs(out64).max(axis=1, keepdims=True), 1e-30)
    assert np.max(np.abs(out32 - out64) / scale) < 1e-5
    xf = (x if w.dtype == workloads.F32 else workloads.bf16_bits_to_f32(x)).reshape(T, G).astype(np.float64)
    err = np.linalg.norm(out64 - xf, axis=1)
    assert np.all(err <= sf / 2 * math.sqrt(G) * (1 + 1e-3) + 1e-6 * np.abs(xf).max(axis=1))
    # fewer levels, larger steps: the INT2/INT3 stream is coarser than INT3/INT4 at the same fraction of wide tiles
    cfg34 = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget + 1.0)
    out34 = o32.decode(cfg34, o32.encode(cfg34, x), o32.F32).astype(np.float64)
    assert np.linalg.norm(out64.reshape(-1) - xf.reshape(-1)) > 1.5 * np.linalg.norm(out34 - xf.reshape(-1))


def test_two_bit_codes_fill_a_quarter_byte_each_in_element_order():
    # one tile, values exactly on the four levels: codes 0..3 repeated, element i at bits [2i, 2i+2)
    G = 32
    x = np.tile(np.array([0.0, 1.0, 2.0, 3.0], np.float32), G // 4).reshape(1, 1, G)
    cfg = o32.make_cfg(1, 1, G, G, o32.F32, 2.0, tau=float("inf"), low_bits=2)
    packed = o32.encode(cfg, x)
    s = o64.parse_stream(packed, 1, G, 1, 0, low=2)
    assert float(s["scale"][0]) == 1.0 and float(s["zero"][0]) == 0.0
    assert np.array_equal(s["codes"][0], np.tile([0, 1, 2, 3], G // 4))
    pay = packed[s["offsets"]["payload"]:]
    assert pay.size == G * 2 // 8 and (pay == 0b11100100).all()
    assert np.array_equal(o32.decode(cfg, packed).reshape(x.shape), x)


# -------------------------------------------------------------- format

def test_packed_size_closed_form_and_expected_sizes():
    # Sec. 3.4: the stream's shape depends on the configuration only.
    want = {1: 38144, 2: 2175040, 3: 13942848, 4: 130809920, 5: 111083584}
    for i, w in enumerate(workloads.CONFIGS, 1):
        cfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
        T = o32.n_tiles(cfg)
        k = o32.k_per_unit(cfg)
        off = o64.section_offsets(T, w.tile, w.batch, k)
        assert o32.packed_size(cfg) == off["total"] == want[i]


def test_wire_cost_close_to_papers_4p41_bits():
    # Sec. 3.4: 80% INT4 + 20% INT3 at A=G=64 -> about 4.41 bits/element of which about 0.61 metadata
    # (39 bits per tile: 16 scale + 16 zero-point + 1 width bit + 6 pivot bits).  This format spends
    # 41.5 bits per tile (byte-aligned pivot with a flag bit, rank table).
    cfg = o32.make_cfg(4, 1024, 4096, 64, o32.BF16, 3.8)
    bits = 8 * (o32.packed_size(cfg) - 64) / (4 * 1024 * 4096)
    assert abs(bits - (3.8 + 41.5 / 64)) < 1e-3
    assert abs(bits - 4.41) < 0.05


def test_invalid_configs_have_size_zero():
    assert o32.packed_size(o32.make_cfg(1, 4, 100, 64, o32.F32, 3.5)) == 0
    assert o32.packed_size(o32.make_cfg(1, 4, 128, 4, o32.F32, 3.5)) == 0
    assert o32.packed_size(o32.make_cfg(1, 4, 144, 48, o32.F32, 3.5)) == 0
    assert o32.packed_size(o32.make_cfg(1, 4, 128, 64, o32.F32, 4.5)) == 0
    assert o32.packed_size(o32.make_cfg(0, 4, 128, 64, o32.F32, 3.5)) == 0


# ------------------------------------------- whole codec, small tensors

def _small_cases():
    yield 1, dict(batch=1, seq=16)
    yield 2, dict(batch=2, seq=24)
    yield 3, dict(batch=2, seq=8)
    yield 4, dict(batch=2, seq=40)
    yield 5, dict(batch=2, seq=16)


@pytest.mark.parametrize("index,shape", list(_small_cases()))
@pytest.mark.parametrize("budget", (None, 3.5))
def test_stream_parses_and_decodes_independently_in_float64(index, shape, budget):
    w, x = workloads.generate(index, **shape)
    budget = w.budget_bits if budget is None else budget
    cfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget)
    packed = o32.encode(cfg, x)
    T, G = o32.n_tiles(cfg), w.tile
    k = o32.k_per_unit(cfg)
    assert packed.size == o32.packed_size(cfg)
    out64, s = o64.decode_stream(packed, T, G, w.batch, k)

    # header
    assert bytes(s["header"][:4]) == b"TAHQ"
    hdr = s["header"].view("<u4")
    assert list(hdr[1:9]) == [1, w.dtype, w.batch, w.seq, w.hidden, G, 0, k]
    assert hdr[9:14].view("<f4").tolist() == [np.float32(budget), 2.0, np.float32(1e-8), np.float32(1e-8), np.float32(1e-8)]

    # bit map: exactly k INT4 tiles per sample, equal to the top-k of the float64-sorted fp32 entropies
    H, pivot, mn, mx = o32.tile_stats(cfg, x)
    assert np.array_equal(s["bits"].reshape(w.batch, -1).sum(axis=1), np.full(w.batch, k))
    assert np.array_equal(s["width"], o64.allocate(H, w.batch, k))
    assert np.array_equal(s["ranks"], s["rank_of"][::64])
    assert np.array_equal(s["pivot"], pivot)

    # every section's padding is zero and the payload is dense
    off = s["offsets"]
    assert not packed[off["bitmap"] + (T + 7) // 8: off["ranks"]].any()
    assert not packed[off["pivot"] + T: off["scale"]].any()

    # metadata covers the range, codes are in range
    sf = s["scale"].astype(np.float64); zf = s["zero"].astype(np.float64)
    L = (1 << s["width"]) - 1
    assert np.all(zf <= mn) and np.all(zf + L * sf >= mx)
    assert np.all(s["codes"] <= L[:, None])

    # float64 decode of the parsed stream agrees with the C decoder
    out32 = o32.decode(cfg, packed, o32.F32).reshape(T, G).astype(np.float64)
    scale = np.maximum(np.abs(out64).max(axis=1, keepdims=True), 1e-30)
    assert np.max(np.abs(out32 - out64) / scale) < 1e-5

    # reconstruction error: half a step per element in the quantized domain, i.e. (sf/2) sqrt(G) in L2
    xf = (x if w.dtype == workloads.F32 else workloads.bf16_bits_to_f32(x)).reshape(T, G).astype(np.float64)
    err = np.linalg.norm(out64 - xf, axis=1)
    assert np.all(err <= sf / 2 * math.sqrt(G) * (1 + 1e-3) + 1e-6 * np.abs(xf).max(axis=1))
    # Assumption 4's form: relative error well below 1
    assert (np.linalg.norm(out64 - xf) / np.linalg.norm(xf)) ** 2 < 0.4


def test_worked_example_one_hot_tile_is_exact():
    # Tile 16*e_d, G=64: flagged, transformed tile is the constant 2, scale degenerate,
    # all codes 0, decode returns exactly 16*e_d.
    G = 64
    for d in (0, 5, 63):
        x = np.zeros((1, 1, G), np.float32); x[0, 0, d] = 16.0
        cfg = o32.make_cfg(1, 1, G, G, o32.F32, 4.0)
        packed = o32.encode(cfg, x)
        s = o64.parse_stream(packed, 1, G, 1, 1)
        assert s["pivot"][0] == 0x80 | d
        assert float(s["zero"][0]) == 2.0 and float(s["scale"][0]) == 1.0
        assert not s["codes"].any()
        assert np.array_equal(o32.decode(cfg, packed).reshape(1, 1, G), x)


def test_spike_size_does_not_change_the_error_of_the_rest():
    # Sec. 3.3: after the swap the pivot sits on the all-ones Hadamard row, a constant offset that the
    # zero-point absorbs: the error on the other entries does not grow with the spike.  Float16 metadata makes the independence approximate.
    G = 64
    rng = np.random.default_rng(12)
    noise = (rng.integers(-64, 65, size=G) / 64.0).astype(np.float32)
    rest = np.arange(G) != 9
    errs, errs_plain = [], []
    for spike in (64.0, 256.0, 1024.0):
        x = noise.copy(); x[9] = spike
        for tau, acc in ((2.0, errs), (float("inf"), errs_plain)):
            cfg = o32.make_cfg(1, 1, G, G, o32.F32, 4.0, tau=tau)
            packed = o32.encode(cfg, x.reshape(1, 1, G))
            s = o64.parse_stream(packed, 1, G, 1, 1)
            assert s["pivot"][0] == ((0x80 | 9) if tau == 2.0 else 0)
            out = o32.decode(cfg, packed)
            acc.append(float(np.abs(out - x)[rest].max()))
    assert max(errs) < 1.5 * min(errs) and max(errs) < 0.2
    # without the transform every small entry collapses onto one level: the error is their whole range
    assert min(errs_plain) > 5 * max(errs)


def test_tau_infinity_is_plain_minmax_group_quantization():
    # App. (tau study): tau = inf never transforms; the codec is then per-group min-max quantization.
    w, x = workloads.generate(2, batch=1, seq=16)
    cfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, 4.0, tau=float("inf"))
    T, G = o32.n_tiles(cfg), w.tile
    s = o64.parse_stream(o32.encode(cfg, x), T, G, 1, o32.k_per_unit(cfg))
    assert not s["pivot"].any()
    tiles = x.reshape(T, G).astype(np.float64)
    sf = s["scale"].astype(np.float64)[:, None]; zf = s["zero"].astype(np.float64)[:, None]
    # textbook quantizer with the (float16, outward-rounded) parameters the stream carries
    pre = (tiles - zf) / sf
    want = np.clip(np.rint(pre), 0, 15)
    near_tie = np.abs(pre - np.floor(pre) - 0.5) < 1e-4
    assert np.array_equal(s["codes"][~near_tie], want[~near_tie].astype(np.uint8))
    # and against the fully float64 textbook quantizer the reconstruction differs by under a step
    q, s64, mn64 = o64.minmax_group_quantize(tiles, 4)
    assert np.all(np.abs((q * s64 + mn64) - (s["codes"] * sf + zf)) <= sf * 1.01)
    # float16 metadata is tight: within one float16 ulp of the exact values
    assert np.all(sf >= s64 * (1 - 1e-6)) and np.all(sf <= s64 * (1 + 2.0 ** -9) + 1e-7)


def test_tau_zero_flags_every_nonzero_tile():
    w, x = workloads.generate(5, batch=1, seq=32)
    cfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, 4.0, tau=0.0)
    H, pivot, mn, mx = o32.tile_stats(cfg, x)
    nonzero = workloads.bf16_bits_to_f32(x).reshape(-1, w.tile).any(axis=1)
    assert np.array_equal((pivot & 0x80) != 0, nonzero)
    assert (~nonzero).sum() > 0


def test_hadamard_lowers_error_on_planted_outlier_tiles():
    # Sec. 3.3 / ablation: on tiles with a planted outlier the transform reduces the error (sanity only).
    rng = np.random.default_rng(13)
    G = 64
    x = rng.standard_normal((1, 64, G)).astype(np.float32)
    x[0, :, 11] = 60.0
    errs = {}
    for tau in (2.0, float("inf")):
        cfg = o32.make_cfg(1, 64, G, G, o32.F32, 3.0, tau=tau)
        out = o32.decode(cfg, o32.encode(cfg, x)).reshape(x.shape)
        errs[tau] = float(((out - x) ** 2).mean())
    assert errs[2.0] < 0.25 * errs[float("inf")]


def test_entropy_guided_allocation_targets_spread_tiles():
    # Sec. 3.2: INT4 goes to the highest-entropy tiles.  Mix flat (uniform) tiles with peaky ones.
    rng = np.random.default_rng(14)
    G = 64
    flat = rng.uniform(-1, 1, size=(32, G)).astype(np.float32)
    peaky = (rng.standard_normal((32, G)) * 0.01).astype(np.float32); peaky[:, 3] = 5.0
    x = np.concatenate([peaky[:16], flat, peaky[16:]]).reshape(1, 64, G)
    cfg = o32.make_cfg(1, 64, G, G, o32.F32, 3.5)
    s = o64.parse_stream(o32.encode(cfg, x), 64, G, 1, 32)
    assert np.array_equal(np.nonzero(s["bits"])[0], np.arange(16, 48))


def test_edge_tiles_roundtrip_and_parse():
    for G in GS:
        tiles = workloads.edge_tiles(G)
        x = tiles.reshape(1, len(tiles), G)
        for budget in (3.0, 3.5, 4.0):
            cfg = o32.make_cfg(1, len(tiles), G, G, o32.F32, budget)
            packed = o32.encode(cfg, x)
            k = o32.k_per_unit(cfg)
            out64, s = o64.decode_stream(packed, len(tiles), G, 1, k)
            assert s["bits"].sum() == k
            out32 = o32.decode(cfg, packed).reshape(len(tiles), G)
            assert np.all(np.isfinite(out32))
            inr = np.abs(tiles).max(axis=1) < 6e4
            sf = s["scale"].astype(np.float64)
            err = np.linalg.norm(out32[inr].astype(np.float64) - tiles[inr].astype(np.float64), axis=1)
            assert np.all(err <= sf[inr] / 2 * math.sqrt(G) * 1.01 + 1e-6 * np.abs(tiles[inr]).max(axis=1) + 1e-30)
            # the all-zero tile and the one-hot tiles come back exactly
            assert not out32[0].any()
            if G == 64:                      # 1/sqrt(64) is exact
                assert np.array_equal(out32[3], tiles[3])
            assert np.allclose(out32[3], tiles[3], rtol=0, atol=1e-5)


def test_bf16_output_is_rne_of_fp32_output():
    import torch
    w, x = workloads.generate(3, batch=1, seq=8)
    cfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.5)
    packed = o32.encode(cfg, x)
    f = o32.decode(cfg, packed, o32.F32)
    h = o32.decode(cfg, packed, o32.BF16)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(h, want)


def test_workload_generators_are_seeded_and_prefix_stable():
    for i in range(1, 6):
        w, a = workloads.generate(i, batch=1, seq=8) if i != 1 else workloads.generate(1)
        _, b = workloads.generate(i, batch=1, seq=8) if i != 1 else workloads.generate(1)
        assert np.array_equal(a, b)
    w2, big = workloads.generate(2, batch=2, seq=16)
    _, small = workloads.generate(2, batch=1, seq=16)
    assert np.array_equal(big[0], small[0])


def test_outlier_threshold_is_strict():
    # Eq. 3: "exceeds" -- a ratio of exactly tau does not trigger the transform
    v = np.zeros(32, np.float32); v[7] = 2.0; v[3] = -1.0
    assert o32.outlier(v, tau=2.0, eps_ratio=0.0) == (False, 7)
    v[7] = np.nextafter(np.float32(2.0), np.float32(3.0))
    assert o32.outlier(v, tau=2.0, eps_ratio=0.0) == (True, 7)


def test_k_gives_the_mean_width_closest_to_the_budget():
    # top-p% with p = budget - 3: among all integer tile counts, k makes 3 + k/n closest to the budget
    rng = np.random.default_rng(15)
    for _ in range(200):
        n_tok = int(rng.integers(1, 40))
        n = n_tok * 3
        budget = float(np.float32(rng.uniform(3.0, 4.0)))
        cfg = o32.make_cfg(1, n_tok, 96, 32, o32.F32, budget)
        k = o32.k_per_unit(cfg)
        gaps = np.abs(3.0 + np.arange(n + 1) / n - budget)
        best = np.nonzero(np.isclose(gaps, gaps.min(), rtol=0, atol=1e-12))[0]
        assert k in best, (n, budget, k, best)
    cfg = o32.make_cfg(1, 4, 96, 32, o32.F32, 3.4)      # n = 12: 0.4 * 12 = 4.8 -> 5 tiles
    assert o32.k_per_unit(cfg) == 5


@pytest.mark.parametrize("low", (1, 2, 3, 4, 5, 6, 7))
def test_any_pair_of_neighbouring_widths(low):
    # the appendix on bit allocation sweeps the ratio of two neighbouring widths (and tries a 2/3-bit mix): widths lo
    # and lo+1 for any lo.  Pinned here: the budget range moves with lo; the mean payload width is the budget; at the
    # ends of the range every tile has one width; codes stay below 2^b; the float64 reading of the stream meets the
    # half-step bound per tile; and at 8 bits a code is a byte of the payload.
    rng = np.random.default_rng(90 + low)
    B, S, G, M = 2, 24, 32, 5
    x = rng.standard_normal((B, S, G * M)).astype(np.float32)
    x[:, :, 7::41] *= 30.0
    T, n = B * S * M, S * M
    assert o32.packed_size(o32.make_cfg(B, S, G * M, G, o32.F32, low - 0.01, low_bits=low)) == 0
    assert o32.packed_size(o32.make_cfg(B, S, G * M, G, o32.F32, low + 1.01, low_bits=low)) == 0
    for budget in (float(low), low + 0.25, low + 0.7, low + 1.0):
        cfg = o32.make_cfg(B, S, G * M, G, o32.F32, budget, tau=float("inf"), low_bits=low)
        k = o32.k_per_unit(cfg)
        assert k == round((budget - low) * n)
        packed = o32.encode(cfg, x)
        out64, s = o64.decode_stream(packed, T, G, B, k, low=low)
        assert set(np.unique(s["width"])) <= {low, low + 1} and int((s["width"] == low + 1).sum()) == B * k
        assert abs(s["width"].mean() - budget) < 1.0 / n
        L = (1 << s["width"]) - 1
        assert np.all(s["codes"] <= L[:, None])
        # untransformed tiles (tau = inf): every element within half a step of its reconstruction
        step = s["scale"].astype(np.float64)[:, None]
        assert np.all(np.abs(out64 - x.reshape(T, G).astype(np.float64)) <= 0.5 * step * (1 + 1e-6))
        assert np.array_equal(o32.decode(cfg, packed, o32.F32).reshape(T, G), out64.astype(np.float32))
    if low == 7:
        off = o64.section_offsets(T, G, B, n, low=7)
        assert np.array_equal(packed[off["payload"]:off["total"]].reshape(T, G), s["codes"].astype(np.uint8))
    assert o32.packed_size(o32.make_cfg(B, S, G * M, G, o32.F32, 8.5, low_bits=8)) == 0
