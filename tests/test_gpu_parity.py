"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: bit-exact entropies (they decide the allocation), bit maps, rank tables, pivots, binary16
metadata, payload bytes -- i.e. the whole stream -- and decoded fp32 output within 1e-6 absolute
(in practice bit-identical), decoded bf16 output bit-identical.
"""
import sys

import numpy as np
import pytest

import workloads
from oracle import o32, o64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def tahq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2506_01352_amd as t
    t.binding._load()          # fail loudly if the HIP library is missing
    return t


def to_device(x):
    """Host array -> device tensor with the same bytes (bf16 bit patterns travel as int16)."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda()
    return torch.from_numpy(x).cuda()


CANARY = 0xA5


class Guarded:
    """A device byte buffer with canary bytes on both sides."""

    def __init__(self, nbytes, pad=256):
        self.pad, self.nbytes = pad, nbytes
        self.raw = torch.full((nbytes + 2 * pad,), CANARY, dtype=torch.uint8, device="cuda")
        self.view = self.raw[pad:pad + nbytes]
        assert self.view.data_ptr() % 16 == 0

    def check(self):
        r = self.raw.cpu().numpy()
        assert (r[:self.pad] == CANARY).all() and (r[self.pad + self.nbytes:] == CANARY).all(), "out-of-bounds write"


def run_gpu(tahq, cfg, x, out_dtype, want_alloc_entropy=False):
    """encode + decode on the GPU with guarded buffers; returns (entropy, packed, out) on the host, plus the
    entropies of the allocation tiles if asked for."""
    d_in = to_device(x)
    n = x.size
    T = n // cfg.tile
    packed = Guarded(tahq.tahq_packed_size(cfg))
    ws = Guarded(tahq.tahq_workspace_size(cfg))
    ent = Guarded(4 * T)
    ent_a = Guarded(4 * (n // (cfg.alloc_tile or cfg.tile)))
    esz = 4 if out_dtype == tahq.F32 else 2
    out = Guarded(esz * n)
    tahq.tahq_tile_entropy(cfg, d_in, ent.view)
    tahq.tahq_alloc_tile_entropy(cfg, d_in, ent_a.view, ws.view)
    ws.view.fill_(0x3C)         # the encoder must not rely on what the call above left behind
    tahq.tahq_encode(cfg, d_in, packed.view, ws.view)
    tahq.tahq_decode(cfg, packed.view, out.view, out_dtype)
    # the same encode with the general multi-launch selection (small ranking units take a single-launch path
    # by default): byte-identical stream
    packed2 = Guarded(tahq.tahq_packed_size(cfg))
    ws.view.fill_(0xC3)
    tahq.tahq_encode_phases(cfg, d_in, packed2.view, ws.view, tahq.PHASE_ALL | tahq.SELECT_MULTI_LAUNCH)
    torch.cuda.synchronize()
    for g in (packed, packed2, ws, ent, ent_a, out):
        g.check()
    assert torch.equal(packed.view, packed2.view), "single-launch and multi-launch selection disagree"
    H = ent.view.cpu().numpy().view(np.float32)
    o = out.view.cpu().numpy().view(np.float32 if out_dtype == tahq.F32 else np.uint16)
    if want_alloc_entropy:
        return H, packed.view.cpu().numpy(), o, ent_a.view.cpu().numpy().view(np.float32)
    return H, packed.view.cpu().numpy(), o


def first_diff(a, b):
    idx = np.nonzero(a != b)[0]
    return None if idx.size == 0 else int(idx[0])


def compare_streams(got, want, T, G, n_units, k, low=3):
    """Byte-exact comparison with a section-by-section report on failure."""
    if np.array_equal(got, want):
        return
    off = o64.section_offsets(T, G, n_units, k, low)
    names = ["bitmap", "ranks", "pivot", "scale", "zero", "payload", "total"]
    report = []
    if not np.array_equal(got[:64], want[:64]):
        report.append("header differs")
    for a, b in zip(names[:-1], names[1:]):
        d = first_diff(got[off[a]:off[b]], want[off[a]:off[b]])
        if d is not None:
            nd = int((got[off[a]:off[b]] != want[off[a]:off[b]]).sum())
            report.append(f"{a}: {nd} bytes differ, first at +{d} (got {got[off[a] + d]:#x}, want {want[off[a] + d]:#x})")
    raise AssertionError("stream mismatch: " + "; ".join(report))


def check_case(tahq, x, B, S, Cc, G, dtype, budget, out_dtype=None, **kw):
    cfg = tahq.make_config(B, S, Cc, G, dtype, budget, **kw)
    ocfg = o32.make_cfg(B, S, Cc, G, dtype, budget, **kw)
    out_dtype = dtype if out_dtype is None else out_dtype
    x = np.ascontiguousarray(x).reshape(B, S, Cc)
    H, packed, out, HA = run_gpu(tahq, cfg, x, out_dtype, want_alloc_entropy=True)
    T = B * S * (Cc // G)
    wantH, _, _, _ = o32.tile_stats(ocfg, x)
    assert np.array_equal(H.view(np.uint32), wantH.view(np.uint32)), \
        f"entropy bits differ at tile {first_diff(H.view(np.uint32), wantH.view(np.uint32))}"
    wantHA = o32.alloc_entropies(ocfg, x)
    assert np.array_equal(HA.view(np.uint32), wantHA.view(np.uint32)), \
        f"allocation-tile entropy bits differ at {first_diff(HA.view(np.uint32), wantHA.view(np.uint32))}"
    want = o32.encode(ocfg, x)
    n_units = 1 if kw.get("scope", 0) else B
    compare_streams(packed, want, T, G, n_units, o32.k_per_unit(ocfg) * o32.tiles_per_alloc(ocfg), o32.low_bits(ocfg))
    want_out = o32.decode(ocfg, want, out_dtype)
    if out_dtype == tahq.F32:
        fin = np.isfinite(want_out)
        assert np.array_equal(np.isfinite(out), fin)
        assert np.all(np.abs(out[fin].astype(np.float64) - want_out[fin].astype(np.float64)) <= 1e-6)
        assert np.array_equal(out.view(np.uint32)[fin], want_out.view(np.uint32)[fin])
    else:
        assert np.array_equal(out, want_out)
    return packed


# ----------------------------------------------------------------- cases

SMALL = [
    # (config index, generator shape): several tiles per block, ragged tails, n not a multiple of 64/512
    (1, dict()),
    (2, dict(batch=2, seq=40)),
    (2, dict(batch=3, seq=7)),
    (3, dict(batch=2, seq=24)),
    (3, dict(batch=1, seq=3)),
    (4, dict(batch=2, seq=36)),
    (5, dict(batch=3, seq=10)),
    (5, dict(batch=2, seq=33)),
]


@pytest.mark.parametrize("index,shape", SMALL)
@pytest.mark.parametrize("budget", (None, 3.0, 3.3, 4.0))
def test_small_workloads_bit_exact(tahq, index, shape, budget):
    w, x = workloads.generate(index, **shape)
    budget = w.budget_bits if budget is None else budget
    _say(f"[case] {w.name} shape={w.batch}x{w.seq}x{w.hidden} budget={budget}")
    check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, budget)


@pytest.mark.parametrize("index,shape", [(2, dict(batch=2, seq=40)), (4, dict(batch=2, seq=36))])
def test_output_dtype_other_than_input(tahq, index, shape):
    w, x = workloads.generate(index, **shape)
    other = tahq.BF16 if w.dtype == tahq.F32 else tahq.F32
    _say(f"[case] {w.name} out_dtype={other}")
    check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.5, out_dtype=other)


@pytest.mark.parametrize("G", (8, 16, 32, 64, 128))
@pytest.mark.parametrize("budget", (3.0, 3.5, 4.0))
def test_edge_tiles(tahq, G, budget):
    tiles = workloads.edge_tiles(G)
    _say(f"[case] edge tiles G={G} budget={budget} n={len(tiles)}")
    # as one token per tile, and as tokens of three tiles (fp32), and in bf16
    n = len(tiles) // 3 * 3
    check_case(tahq, tiles, 1, len(tiles), G, G, tahq.F32, budget)
    check_case(tahq, tiles[:n], 1, n // 3, 3 * G, G, tahq.F32, budget)
    check_case(tahq, workloads.f32_to_bf16_bits(tiles), 1, len(tiles), G, G, tahq.BF16, budget)


@pytest.mark.parametrize("tau", (0.0, 4.0, float("inf")))
def test_tau_special_cases(tahq, tau):
    w, x = workloads.generate(4, batch=1, seq=20)
    _say(f"[case] tau={tau}")
    check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.5, tau=tau)


def test_whole_tensor_ranking_scope(tahq):
    w, x = workloads.generate(2, batch=3, seq=20)
    _say("[case] scope=1")
    check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.4, scope=1)


def test_large_units_with_ties_at_the_threshold(tahq):
    # Ranking units of 65536 and 49152 tiles take the two-launch selection of large units: a histogram of the
    # entropies, then an exact ranking of the tiles in the threshold bin only.  (a) two kinds of token, all tiles of a
    # token alike: the threshold bin holds half a unit, more than the candidate list takes, and thousands of equal
    # entropies are split by tile index; (b) a fifth of the tiles share the highest entropy and the budget cuts that
    # group in two: the list holds them all, the tie is resolved by a second selection on the index; (c) random
    # tiles drawn from a pool of 3000, so that a few equal entropies meet at the threshold; (d) whole-tensor ranking.
    rng = np.random.default_rng(21)
    S, Cc, G = 512, 8192, 64
    pat = rng.standard_normal((2, G)).astype(np.float32)
    pat[1, 5] *= 30.0
    kind = rng.integers(0, 2, size=(2, S))
    xa = np.tile(pat[kind], (1, 1, Cc // G))
    _say("[case] large units, massive ties: list overflow")
    check_case(tahq, workloads.f32_to_bf16_bits(xa), 2, S, Cc, G, tahq.BF16, 3.25)
    check_case(tahq, workloads.f32_to_bf16_bits(xa), 2, S, Cc, G, tahq.BF16, 3.75)

    tiles = rng.standard_normal((2 * S * (Cc // G), G)).astype(np.float32)
    flat = rng.random(tiles.shape[0]) < 0.2
    tiles[flat] = np.where(rng.random((int(flat.sum()), G)) < 0.5, -1.5, 1.5).astype(np.float32)   # entropy ln G
    _say("[case] large units, a fifth of the tiles tied at the top")
    check_case(tahq, workloads.f32_to_bf16_bits(tiles), 2, S, Cc, G, tahq.BF16, 3.1)

    pool = rng.standard_normal((3000, G)).astype(np.float32)
    xc = pool[rng.integers(0, 3000, size=3 * 384 * (Cc // G))]
    _say("[case] large units, tiles from a pool")
    check_case(tahq, xc, 3, 384, Cc, G, tahq.F32, 3.4)
    _say("[case] large units, whole-tensor ranking")
    check_case(tahq, xc, 3, 384, Cc, G, tahq.F32, 3.6, scope=1)


# Sec. 3.2 with allocation tiles of several quantization tiles, up to the whole token (A = C)
WIDE = [
    (1, dict(), 128), (1, dict(), 512),
    (2, dict(batch=2, seq=40), 256), (2, dict(batch=2, seq=40), 2048), (2, dict(batch=3, seq=7), 128),
    (3, dict(batch=2, seq=24), 512), (3, dict(batch=2, seq=24), 4096),
    (4, dict(batch=2, seq=36), 512), (4, dict(batch=2, seq=36), 8192), (4, dict(batch=1, seq=130), 8192),
    (5, dict(batch=3, seq=10), 160), (5, dict(batch=2, seq=33), 5120), (5, dict(batch=2, seq=33), 64),
]


@pytest.mark.parametrize("index,shape,A", WIDE)
def test_allocation_tiles_of_several_quantization_tiles(tahq, index, shape, A):
    w, x = workloads.generate(index, **shape)
    for budget in (3.3, 3.0, 4.0):
        _say(f"[case] {w.name} shape={w.batch}x{w.seq}x{w.hidden} A={A} budget={budget}")
        check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, budget, alloc_tile=A)
    check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, 3.6, alloc_tile=A, scope=1)


@pytest.mark.parametrize("G", (32, 64, 128))
def test_allocation_tiles_of_three_edge_tiles(tahq, G):
    tiles = workloads.edge_tiles(G)
    n = len(tiles) // 3 * 3
    _say(f"[case] edge tiles G={G} A={3 * G}")
    check_case(tahq, tiles[:n], 1, n // 3, 3 * G, G, tahq.F32, 3.5, alloc_tile=3 * G)
    check_case(tahq, workloads.f32_to_bf16_bits(tiles[:n]), n // 3, 1, 3 * G, G, tahq.BF16, 3.5, alloc_tile=3 * G)


def test_allocation_tile_ties_and_many_small_units(tahq):
    # all-zero tokens give allocation tiles of entropy exactly 0; 300 samples of 3 allocation tiles each
    w, x = workloads.generate(5, batch=2, seq=64)
    _say("[case] allocation-tile ties")
    for budget in (3.1, 3.9):
        check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, budget, alloc_tile=640)
    rng = np.random.default_rng(6)
    y = rng.standard_normal((300, 3, 128)).astype(np.float32)
    y[:, :, 17] *= 12.0
    check_case(tahq, y, 300, 3, 128, 64, tahq.F32, 3.34, alloc_tile=128)


# the INT2/INT3 mix of the appendix on bit allocation (low_bits = 2)
@pytest.mark.parametrize("index,shape", SMALL)
@pytest.mark.parametrize("budget", (2.2, 2.0, 3.0))
def test_int2_int3_mix_bit_exact(tahq, index, shape, budget):
    w, x = workloads.generate(index, **shape)
    _say(f"[case] {w.name} shape={w.batch}x{w.seq}x{w.hidden} INT2/INT3 budget={budget}")
    check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, budget, low_bits=2)


@pytest.mark.parametrize("G", (8, 16, 32, 64, 128))
def test_int2_int3_edge_tiles_other_output_type_and_allocation_tiles(tahq, G):
    tiles = workloads.edge_tiles(G)
    n = len(tiles) // 3 * 3
    _say(f"[case] INT2/INT3 edge tiles G={G}")
    for budget in (2.0, 2.5, 3.0):
        check_case(tahq, tiles, 1, len(tiles), G, G, tahq.F32, budget, low_bits=2)
        check_case(tahq, workloads.f32_to_bf16_bits(tiles), 1, len(tiles), G, G, tahq.BF16, budget, out_dtype=tahq.F32,
                   low_bits=2)
    check_case(tahq, tiles[:n], 1, n // 3, 3 * G, G, tahq.F32, 2.4, out_dtype=tahq.BF16, low_bits=2, alloc_tile=3 * G)
    check_case(tahq, tiles[:n], 1, n // 3, 3 * G, G, tahq.F32, 2.4, low_bits=2, scope=1, tau=4.0)


# any pair of neighbouring widths, 1/2 bits up to 7/8 bits (the appendix on bit allocation sweeps the ratio of two widths)
@pytest.mark.parametrize("low", (1, 4, 5, 6, 7))
def test_other_width_pairs_bit_exact(tahq, low):
    for index, shape in ((2, dict(batch=2, seq=40)), (4, dict(batch=2, seq=36)), (3, dict(batch=2, seq=24)),
                         (5, dict(batch=3, seq=10)), (1, dict())):
        w, x = workloads.generate(index, **shape)
        for budget in (low + 0.3, float(low), low + 1.0):
            _say(f"[case] {w.name} shape={w.batch}x{w.seq}x{w.hidden} widths {low}/{low + 1} budget={budget}")
            check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, budget, low_bits=low)
    # edge tiles at every tile width, the other output type, an allocation tile of three tiles, whole-tensor ranking
    for G in (8, 16, 32, 64, 128):
        tiles = workloads.edge_tiles(G)
        n = len(tiles) // 3 * 3
        _say(f"[case] widths {low}/{low + 1} edge tiles G={G}")
        check_case(tahq, tiles, 1, len(tiles), G, G, tahq.F32, low + 0.5, low_bits=low)
        check_case(tahq, workloads.f32_to_bf16_bits(tiles), 1, len(tiles), G, G, tahq.BF16, low + 0.5,
                   out_dtype=tahq.F32, low_bits=low)
        check_case(tahq, tiles[:n], 1, n // 3, 3 * G, G, tahq.F32, low + 0.4, out_dtype=tahq.BF16, low_bits=low,
                   alloc_tile=3 * G)
        check_case(tahq, tiles[:n], 1, n // 3, 3 * G, G, tahq.F32, low + 0.4, low_bits=low, scope=1, tau=4.0)


def test_massive_entropy_ties_are_broken_by_index(tahq):
    # config-5-like tensor (20% all-zero tokens: entropy exactly 0) with a budget that puts the
    # threshold inside the tie, plus a tensor whose tiles are all identical
    w, x = workloads.generate(5, batch=2, seq=64)
    _say("[case] ties at the threshold")
    for budget in (3.1, 3.85, 3.95):
        check_case(tahq, x, w.batch, w.seq, w.hidden, w.tile, w.dtype, budget)
    rng = np.random.default_rng(0)
    row = rng.standard_normal(64).astype(np.float32)
    same = np.tile(row, (2, 50, 8))
    check_case(tahq, same, 2, 50, 512, 64, tahq.F32, 3.37)


def test_single_tile_and_tiny_tensors(tahq):
    rng = np.random.default_rng(1)
    for G in (8, 16, 32, 64, 128):
        for B, S, M in ((1, 1, 1), (1, 1, 2), (2, 1, 1), (1, 5, 3)):
            x = rng.standard_normal((B, S, M * G)).astype(np.float32)
            x[..., 3] *= 25
            _say(f"[case] tiny G={G} {B}x{S}x{M * G}")
            for budget in (3.0, 3.5, 4.0):
                check_case(tahq, x, B, S, M * G, G, tahq.F32, budget)


def test_repeated_calls_are_deterministic_and_workspace_contents_do_not_matter(tahq):
    w, x = workloads.generate(4, batch=2, seq=64)
    cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
    d_in = to_device(x)
    packed = torch.empty(tahq.tahq_packed_size(cfg), dtype=torch.uint8, device="cuda")
    ws = torch.empty(tahq.tahq_workspace_size(cfg), dtype=torch.uint8, device="cuda")
    results = []
    for fill in (0, 0xFF, 0x5A):
        ws.fill_(fill)
        packed.fill_(0xEE)
        tahq.tahq_encode(cfg, d_in, packed, ws)
        torch.cuda.synchronize()
        results.append(packed.cpu().numpy().copy())
    assert np.array_equal(results[0], results[1]) and np.array_equal(results[1], results[2])


def test_phase_by_phase_calls_write_the_same_stream(tahq):
    # tahq_encode_phases, one phase per call, against the one call: uniform widths (the one call folds the constant
    # bit map into its first kernel, a call for the selection phase alone writes it by itself), small ranking units,
    # large ranking units
    cases = [(3, dict(batch=2, seq=64), None), (3, dict(batch=2, seq=64), 4.0), (2, dict(batch=2, seq=64), None),
             (4, dict(batch=1, seq=1024), None)]
    for index, shape, budget in cases:
        w, x = workloads.generate(index, **shape)
        budget = w.budget_bits if budget is None else budget
        _say(f"[case] phases one by one, {w.name} budget {budget}")
        cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget)
        d_in = to_device(x)
        whole = Guarded(tahq.tahq_packed_size(cfg))
        parts = Guarded(tahq.tahq_packed_size(cfg))
        ws = Guarded(tahq.tahq_workspace_size(cfg))
        ws.view.fill_(0x77)
        tahq.tahq_encode(cfg, d_in, whole.view, ws.view)
        ws.view.fill_(0x11)
        for phase in (tahq.PHASE_PROLOGUE, tahq.PHASE_ENTROPY, tahq.PHASE_SELECT, tahq.PHASE_QUANT):
            tahq.tahq_encode_phases(cfg, d_in, parts.view, ws.view, phase)
        torch.cuda.synchronize()
        for g in (whole, parts, ws):
            g.check()
        assert torch.equal(whole.view, parts.view)
        ocfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, budget)
        assert np.array_equal(whole.view.cpu().numpy(), o32.encode(ocfg, x))


def test_side_stream(tahq):
    w, x = workloads.generate(2, batch=1, seq=64)
    cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
    ocfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
    d_in = to_device(x)
    codec = tahq.Codec(cfg, out_dtype=tahq.F32)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        codec.encode(d_in, stream=s)
        codec.decode(stream=s)
    s.synchronize()
    want = o32.encode(ocfg, x)
    assert np.array_equal(codec.packed.cpu().numpy(), want)
    assert np.array_equal(codec.out.cpu().numpy(), o32.decode(ocfg, want))


# ------------------------------------------------------- full-size configs

@pytest.mark.parametrize("index", (1, 2, 3, 5, 4))
def test_full_size_configs_bit_exact(tahq, index):
    w, x = workloads.generate(index)
    _say(f"[case] full size {w.name}: generated")
    cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
    ocfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits)
    d_in = to_device(x)
    codec = tahq.Codec(cfg)                      # decode into the input dtype, as the benchmark does
    T = w.elements // w.tile
    ent = torch.empty(T, dtype=torch.float32, device="cuda")
    tahq.tahq_tile_entropy(cfg, d_in, ent)
    codec.encode(d_in)
    codec.decode()
    torch.cuda.synchronize()
    _say("[case]   gpu done; oracle encode ...")
    want = o32.encode(ocfg, x)
    _say("[case]   oracle encode done")
    compare_streams(codec.packed.cpu().numpy(), want, T, w.tile, w.batch, o32.k_per_unit(ocfg))
    wantH, _, _, _ = o32.tile_stats(ocfg, x)
    assert np.array_equal(ent.cpu().numpy().view(np.uint32), wantH.view(np.uint32))
    _say("[case]   oracle decode ...")
    want_out = o32.decode(ocfg, want, w.dtype)
    got = codec.out.cpu()
    got = got.numpy() if w.dtype == tahq.F32 else got.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got.view(np.uint32 if w.dtype == tahq.F32 else np.uint16),
                          want_out.view(np.uint32 if w.dtype == tahq.F32 else np.uint16))


def test_full_size_int2_int3_mix_bit_exact(tahq):
    # the headline tensor at 80% INT2 + 20% INT3 (the appendix's setting)
    w, x = workloads.generate(4)
    d_in = to_device(x)
    T = w.elements // w.tile
    _say(f"[case] full size {w.name} INT2/INT3 budget 2.2")
    cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, 2.2, low_bits=2)
    ocfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, 2.2, low_bits=2)
    codec = tahq.Codec(cfg)
    codec.encode(d_in)
    codec.decode()
    torch.cuda.synchronize()
    want = o32.encode(ocfg, x)
    compare_streams(codec.packed.cpu().numpy(), want, T, w.tile, w.batch, o32.k_per_unit(ocfg), 2)
    want_out = o32.decode(ocfg, want, w.dtype)
    got = codec.out.cpu().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want_out)


@pytest.mark.parametrize("G", (8, 16))
def test_one_full_sample_in_small_tiles_bit_exact(tahq, G):
    # one sample of the headline tensor cut into tiles of 8 / 16 channels: 4.2 M / 2.1 M tiles, thousands of batches
    w, x = workloads.generate(4, batch=1)
    _say(f"[case] {w.name} one sample, G={G}")
    cfg = tahq.make_config(1, w.seq, w.hidden, G, w.dtype, w.budget_bits)
    ocfg = o32.make_cfg(1, w.seq, w.hidden, G, w.dtype, w.budget_bits)
    codec = tahq.Codec(cfg)
    codec.encode(to_device(x))
    codec.decode()
    torch.cuda.synchronize()
    want = o32.encode(ocfg, x)
    compare_streams(codec.packed.cpu().numpy(), want, x.size // G, G, 1, o32.k_per_unit(ocfg))
    got = codec.out.cpu().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, o32.decode(ocfg, want, w.dtype))


def test_full_size_token_level_allocation_bit_exact(tahq):
    # the headline tensor with A = C (Sec. 3.2's token-level special case) and with A = 2G
    w, x = workloads.generate(4)
    d_in = to_device(x)
    T = w.elements // w.tile
    for A in (w.hidden, 2 * w.tile):
        _say(f"[case] full size {w.name} A={A}")
        cfg = tahq.make_config(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits, alloc_tile=A)
        ocfg = o32.make_cfg(w.batch, w.seq, w.hidden, w.tile, w.dtype, w.budget_bits, alloc_tile=A)
        codec = tahq.Codec(cfg)
        codec.encode(d_in)
        codec.decode()
        torch.cuda.synchronize()
        want = o32.encode(ocfg, x)
        compare_streams(codec.packed.cpu().numpy(), want, T, w.tile, w.batch, o32.k_per_unit(ocfg) * (A // w.tile))
        want_out = o32.decode(ocfg, want, w.dtype)
        got = codec.out.cpu().view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got, want_out)
        del codec


# ------------------------------------- every (tile width, dtype) pair, several batches and a ragged tail

@pytest.mark.parametrize("G", (8, 16, 32, 64, 128))
@pytest.mark.parametrize("dtype_name", ("f32", "bf16"))
def test_all_tile_widths_and_dtypes_over_several_batches(tahq, G, dtype_name):
    # a workgroup handles min(256, 32768 / tile bytes) tiles: take 3 full batches plus a ragged tail, with
    # sample boundaries that fall inside batches
    dtype = tahq.F32 if dtype_name == "f32" else tahq.BF16
    tile_bytes = G * (4 if dtype == tahq.F32 else 2)
    tiles_per_batch = min(256, 32768 // tile_bytes)
    M = 3
    S = (3 * tiles_per_batch + 37) // M
    B = 2
    rng = np.random.default_rng(G + (7 if dtype == tahq.F32 else 11))
    x = rng.standard_normal((B, S, M * G)).astype(np.float32)
    x[:, :, 5] *= 30.0
    x[:, ::7, :] = rng.uniform(-8, 8, size=x[:, ::7, :].shape).astype(np.float32)
    x[1, 3:9, :] = 0.0
    xin = x if dtype == tahq.F32 else workloads.f32_to_bf16_bits(x)
    for budget in (3.3, 4.0):
        _say(f"[case] G={G} {dtype_name} shape={B}x{S}x{M * G} budget={budget}")
        check_case(tahq, xin, B, S, M * G, G, dtype, budget)
        check_case(tahq, xin, B, S, M * G, G, dtype, budget,
                   out_dtype=(tahq.BF16 if dtype == tahq.F32 else tahq.F32))


@pytest.mark.parametrize("G", (8, 16, 32, 64))
def test_hidden_size_1600_and_small_tiles_on_a_workload(tahq, G):
    # 1600 channels: 200 / 100 / 50 / 25 tiles per token, sample boundaries inside batches and 64-tile groups
    rng = np.random.default_rng(60 + G)
    x = rng.standard_normal((3, 11, 1600)).astype(np.float32)
    x[:, :, 7::53] *= 30.0
    x[2, 4:6, :] = 0.0
    for dtype, xin in ((tahq.F32, x), (tahq.BF16, workloads.f32_to_bf16_bits(x))):
        _say(f"[case] hidden 1600 G={G} dtype={dtype}")
        check_case(tahq, xin, 3, 11, 1600, G, dtype, 3.8)
        check_case(tahq, xin, 3, 11, 1600, G, dtype, 2.2, low_bits=2)
    check_case(tahq, x, 3, 11, 1600, G, tahq.F32, 3.4, alloc_tile=1600)
    # configuration 4's tokens cut into tiles of G channels
    w, y = workloads.generate(4, batch=2, seq=6)
    check_case(tahq, y, w.batch, w.seq, w.hidden, G, w.dtype, w.budget_bits)


@pytest.mark.parametrize("B,S,Cc,G", [(1, 1000, 1600, 64), (2, 1024, 1024, 32), (1, 700, 4096, 64), (1, 513, 2048, 32),
                                       (3, 1024, 1024, 64), (2, 260, 8064, 64)])
def test_ranking_units_of_every_single_launch_size(tahq, B, S, Cc, G):
    # units of 25000 / 32768 / 44800 / 32832 / 16384 / 32760 tiles: every keys-per-thread variant of the single-launch
    # selection, aligned and not aligned to 64 tiles, with all-zero tokens (massive ties) and near-constant tokens
    rng = np.random.default_rng(B * S + Cc + G)
    x = rng.standard_normal((B, S, Cc)).astype(np.float32)
    x[:, :, 3::97] *= 20.0
    x[:, ::9, :] = 0.0                                   # ties at entropy 0
    x[:, 1::13, :] = 1.5                                 # ties at entropy ln G
    _say(f"[case] single-launch selection: units of {S * (Cc // G)} tiles, {B}x{S}x{Cc} G={G}")
    for budget in (3.07, 3.5, 3.93):
        check_case(tahq, workloads.f32_to_bf16_bits(x), B, S, Cc, G, tahq.BF16, budget)
    check_case(tahq, x, B, S, Cc, G, tahq.F32, 3.3, scope=1 if B * S * (Cc // G) <= 65536 else 0)


def test_many_ranking_units_with_few_tiles_each(tahq):
    # 300 samples of 6 tiles: units smaller than a wavefront, a batch spans many units
    rng = np.random.default_rng(5)
    x = rng.standard_normal((300, 2, 192)).astype(np.float32)
    x[:, :, 17] *= 12.0
    _say("[case] 300 units x 6 tiles")
    for budget in (3.34, 3.5, 3.67):
        check_case(tahq, x, 300, 2, 192, 64, tahq.F32, budget)


def test_nan_inf_and_huge_inputs_are_lossy_but_never_a_fault(tahq):
    # Outside the contract: the result for the poisoned sample is unspecified, but nothing may fault or hang,
    # and a clean sample in the same tensor must still match the oracle bit for bit (ranking is per sample).
    rng = np.random.default_rng(9)
    G, S, M = 64, 40, 8
    x = rng.standard_normal((2, S, M * G)).astype(np.float32)
    x[:, :, 11] *= 25.0
    clean = x[1:2].copy()
    x[0, 0, 3] = np.nan
    x[0, 1, 70] = np.inf
    x[0, 2, 130] = -np.inf
    x[0, 3, :64] = 3e38
    x[0, 4, 64:128] = np.nan
    x[0, 5, 200] = 1e30
    for dtype, conv in ((tahq.F32, lambda a: a), (tahq.BF16, workloads.f32_to_bf16_bits)):
        _say(f"[case] non-finite inputs dtype={dtype}")
        with np.errstate(all="ignore"):
            xin = np.ascontiguousarray(conv(x))
        cfg = tahq.make_config(2, S, M * G, G, dtype, 3.5)
        H, packed, out = run_gpu(tahq, cfg, xin, tahq.F32)
        # the clean sample alone, through the oracle
        ocfg1 = o32.make_cfg(1, S, M * G, G, dtype, 3.5)
        want = o32.encode(ocfg1, np.ascontiguousarray(conv(clean)))
        n, k = S * M, o32.k_per_unit(ocfg1)
        T = 2 * n
        off2 = o64.section_offsets(T, G, 2, k)
        off1 = o64.section_offsets(n, G, 1, k)
        # per-tile sections of sample 1 sit at tile offset n
        assert np.array_equal(packed[off2["pivot"] + n: off2["pivot"] + 2 * n], want[off1["pivot"]: off1["pivot"] + n])
        assert np.array_equal(packed[off2["scale"] + 2 * n: off2["scale"] + 4 * n], want[off1["scale"]: off1["scale"] + 2 * n])
        assert np.array_equal(packed[off2["zero"] + 2 * n: off2["zero"] + 4 * n], want[off1["zero"]: off1["zero"] + 2 * n])
        assert np.array_equal(packed[off2["bitmap"] + n // 8: off2["bitmap"] + 2 * n // 8],
                              want[off1["bitmap"]: off1["bitmap"] + n // 8])
        pay1 = (G // 8) * (3 * n + k)
        assert np.array_equal(packed[off2["payload"] + pay1: off2["total"]], want[off1["payload"]: off1["total"]])
        want_out = o32.decode(ocfg1, want, o32.F32)
        assert np.array_equal(out[n * G:].view(np.uint32), want_out.view(np.uint32))


def test_non_finite_entropies_in_large_ranking_units_follow_key_order(tahq):
    # NaN and infinite inputs give NaN entropies; the selection orders tiles by their entropies' order-preserving keys,
    # where a NaN with the sign bit clear sorts above +infinity.  The two-launch selection of large units (bins of
    # the entropy) and the multi-launch radix select (digits of the key) must agree on such a tensor too; run_gpu
    # compares their streams.  The clean sample is checked against the oracle.
    rng = np.random.default_rng(19)
    G, S, M = 32, 1024, 64                          # 65536 tiles per sample: above the single-launch limit
    x = rng.standard_normal((2, S, M * G)).astype(np.float32)
    clean = x[1:2].copy()
    x[0, 0, 3] = np.nan
    x[0, 7, 70] = np.inf
    x[0, 9, 130] = -np.inf
    x[0, 100:140, 64:128] = np.nan
    x[0, 200:260, :32] = 3e38
    x[0, 300:310, :] = 0.0
    for budget in (3.02, 3.5, 3.98):
        _say(f"[case] non-finite inputs, large ranking units, budget {budget}")
        cfg = tahq.make_config(2, S, M * G, G, tahq.F32, budget)
        H, packed, out = run_gpu(tahq, cfg, x, tahq.F32)
        ocfg1 = o32.make_cfg(1, S, M * G, G, tahq.F32, budget)
        want = o32.encode(ocfg1, clean)
        n, k = S * M, o32.k_per_unit(ocfg1)
        off2 = o64.section_offsets(2 * n, G, 2, k)
        off1 = o64.section_offsets(n, G, 1, k)
        assert np.array_equal(packed[off2["bitmap"] + n // 8: off2["bitmap"] + 2 * n // 8],
                              want[off1["bitmap"]: off1["bitmap"] + n // 8])
        pay1 = (G // 8) * (3 * n + k)
        assert np.array_equal(packed[off2["payload"] + pay1: off2["total"]], want[off1["payload"]: off1["total"]])


@pytest.mark.parametrize("G,low", [(64, 3), (32, 2), (8, 3), (128, 3), (16, 2), (64, 7), (16, 5), (128, 1)])
def test_decoding_a_damaged_stream_stays_inside_its_buffers(tahq, G, low):
    # The decoder clamps the rank table to the number of wide tiles the configuration implies, ignores a decreasing
    # table, and masks the pivot index, so every address it forms lies inside the stream and the output whatever
    # bytes arrive.  The values decoded from such a stream are meaningless; the buffers around them must be intact.
    rng = np.random.default_rng(70 + G)
    B, S, Cc = 2, 37, 5 * G * 3                       # several workgroups' batches and a ragged tail
    cfg = tahq.make_config(B, S, Cc, G, tahq.BF16, low + 0.4, low_bits=low)
    size = tahq.tahq_packed_size(cfg)
    T = B * S * (Cc // G)
    off = o64.section_offsets(T, G, B, tahq.tahq_k_per_unit(cfg), low)
    streams = {"random bytes": rng.integers(0, 256, size=size, dtype=np.uint8)}
    ones = np.full(size, 0xFF, np.uint8)
    streams["all ones"] = ones
    z = np.zeros(size, np.uint8)
    z[off["ranks"]:off["pivot"]] = 0xFF               # a rank table far beyond the payload
    z[off["bitmap"]:off["ranks"]] = 0xFF              # every tile claims to be wide
    z[off["pivot"]:off["scale"]] = 0xFF               # every pivot index out of range
    streams["hostile metadata"] = z
    dec = rng.integers(0, 256, size=size, dtype=np.uint8)
    table = dec[off["ranks"]:off["ranks"] + 4 * ((T + 63) // 64)].view("<u4")
    table[:] = np.arange(table.size, 0, -1, dtype=np.uint32)          # a decreasing table
    streams["decreasing rank table"] = dec
    for name, host in streams.items():
        for out_dtype in (tahq.F32, tahq.BF16):
            _say(f"[case] damaged stream G={G} low={low}: {name}, out dtype {out_dtype}")
            packed = Guarded(size)
            packed.view.copy_(torch.from_numpy(host).cuda())
            out = Guarded((4 if out_dtype == tahq.F32 else 2) * B * S * Cc)
            tahq.tahq_decode(cfg, packed.view, out.view, out_dtype)
            torch.cuda.synchronize()
            out.check()
            packed.check()
            assert np.array_equal(packed.view.cpu().numpy(), host)     # the stream is only read


def _large_unit_cases(count, seed):
    """Ranking units above the single-launch limit that start on 64-tile boundaries (the two-launch selection from the
    entropy kernel's histogram), with data that crowds or overflows the threshold bin."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        G = int(rng.choice([8, 16, 32, 64, 128]))
        M = int(rng.choice([16, 32, 64, 128, 40, 24]))
        S = int(rng.choice([512, 1024, 2048, 4096, 768, 1536]))
        B = int(rng.choice([1, 2, 3]))
        n = S * M
        if n <= 32768 or n % 256 or B * n * G > 12_000_000:
            continue
        low = int(rng.choice([3, 3, 3, 2, 4]))
        out.append(dict(B=B, S=S, M=M, G=G, dtype=int(rng.integers(0, 2)), low=low, scope=int(rng.random() < 0.2),
                        budget=float(np.float32(low + rng.uniform(0.02, 0.98))), kind=len(out) % 4,
                        seed=int(rng.integers(0, 2 ** 31))))
    return out


@pytest.mark.parametrize("c", _large_unit_cases(12, seed=5),
                         ids=lambda c: "{B}x{S}x{M}_g{G}_d{dtype}_lo{low}_k{kind}_s{scope}".format(**c))
def test_large_ranking_units_bit_exact(tahq, c):
    rng = np.random.default_rng(c["seed"])
    B, S, Cc, G = c["B"], c["S"], c["M"] * c["G"], c["G"]
    x = rng.standard_normal((B, S, Cc)).astype(np.float32)
    if c["kind"] == 1:      # seven distinct tiles: every entropy is tied thousands of times
        proto = rng.standard_normal((7, G)).astype(np.float32)
        x = proto[rng.integers(0, 7, size=(B, S, c["M"]))].reshape(B, S, Cc)
    elif c["kind"] == 2:    # ties at entropy 0 and at ln G
        x[:, ::3, :] = 0.0
        x[:, 1::5, :] = 1.5
    elif c["kind"] == 3:    # a narrow band of entropies: a crowded threshold bin
        x = (1.0 + 1e-3 * rng.standard_normal((B, S, Cc))).astype(np.float32)
    xin = x if c["dtype"] == 0 else workloads.f32_to_bf16_bits(x)
    _say(f"[case] large ranking units {c}")
    check_case(tahq, xin, B, S, Cc, G, c["dtype"], c["budget"], low_bits=c["low"], scope=c["scope"])


def _random_configurations(count, seed):
    """Seeded sweep over the configuration space: tile width, dtype, widths, budget, allocation tile, scope,
    tau, shapes with ragged batches and ranking units on both sides of the single-launch threshold."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        G = int(rng.choice([8, 16, 32, 64, 128]))
        M = int(rng.choice([1, 2, 3, 5, 8, 12, 25]))                 # tiles per token
        Cc = G * M
        B = int(rng.choice([1, 2, 3, 5]))
        S = int(rng.choice([1, 3, 17, 64, 200, 513, 1500]))
        if B * S * Cc > 6_000_000:
            continue
        low = int(rng.choice([3, 3, 2, 1, 4, 5, 6, 7]))
        budget = float(np.float32(low + rng.choice([0.0, 1.0, rng.uniform(0.02, 0.98)])))
        divisors = [d for d in range(1, M + 1) if M % d == 0]
        m = int(rng.choice(divisors)) if rng.random() < 0.4 else 1
        out.append(dict(B=B, S=S, Cc=Cc, G=G, dtype=int(rng.integers(0, 2)), budget=budget, low_bits=low,
                        alloc_tile=G * m if m > 1 else 0, scope=int(rng.random() < 0.25),
                        tau=float(rng.choice([2.0, 2.0, 1.25, 6.0])), out_dtype=int(rng.integers(0, 2)),
                        data_seed=int(rng.integers(0, 2 ** 31))))
    return out


@pytest.mark.parametrize("case", _random_configurations(120, seed=2024), ids=lambda c: "{B}x{S}x{Cc}_g{G}_d{dtype}_lo{low_bits}_a{alloc_tile}_s{scope}".format(**c))
def test_random_configurations_bit_exact(tahq, case):
    c = case
    rng = np.random.default_rng(c["data_seed"])
    x = rng.standard_normal((c["B"], c["S"], c["Cc"])).astype(np.float32)
    x *= np.exp(rng.standard_normal((c["B"], c["S"], 1))).astype(np.float32)        # token scales
    x[:, :, ::max(1, c["Cc"] // 7)] *= 30.0                                           # outlier channels
    if c["S"] > 4:
        x[:, ::5, :] = 0.0                                                            # ties at entropy 0
        x[:, 1::7, :] = -2.5                                                          # ties at entropy ln G
    xin = x if c["dtype"] == 0 else workloads.f32_to_bf16_bits(x)
    _say(f"[case] random configuration {c}")
    check_case(tahq, xin, c["B"], c["S"], c["Cc"], c["G"], c["dtype"], c["budget"], out_dtype=c["out_dtype"],
               low_bits=c["low_bits"], alloc_tile=c["alloc_tile"], scope=c["scope"], tau=c["tau"])
