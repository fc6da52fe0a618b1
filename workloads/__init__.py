"""Seeded synthetic activation tensors, one recipe per benchmark configuration.

This module serves both the CPU oracle's tests and the HIP path's tests/benchmark.
It holds none of the codec's arithmetic: only random draws, scaling of channels
and tokens, and the fp32 -> bf16 storage conversion of the finished tensor.

The tensors stand in for stage-boundary activations of GPT-style / LLaMA-style
models (hidden 512..8192, sequence 128..4096) and, for the last one, for an
activation-gradient tensor; no dataset or checkpoint is involved.

Every recipe draws, in this order, from numpy.random.Generator(PCG64(seed)):
the per-tensor structure first (outlier channel indices and gains), then sample
after sample.  A tensor generated with a smaller `batch` is therefore a prefix
of the full one.  bf16 tensors are returned as uint16 bit patterns (round to
nearest even); exact zeros are assigned, never produced by multiplying.
"""
from dataclasses import dataclass

import numpy as np

F32, BF16 = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: int        # F32 or BF16
    batch: int
    seq: int
    hidden: int
    tile: int
    budget_bits: float
    seed: int

    @property
    def elements(self):
        return self.batch * self.seq * self.hidden

    @property
    def bytes_per_element(self):
        return 4 if self.dtype == F32 else 2

    def with_shape(self, batch=None, seq=None):
        return Workload(self.name, self.dtype, batch or self.batch, seq or self.seq, self.hidden,
                        self.tile, self.budget_bits, self.seed)


CONFIGS = (
    Workload("cfg1_f32_1x128x512_g64_b4.0", F32, 1, 128, 512, 64, 4.0, 0),
    Workload("cfg2_f32_4x512x2048_g64_b3.5", F32, 4, 512, 2048, 64, 3.5, 1),
    Workload("cfg3_bf16_8x1024x4096_g128_b3.0", BF16, 8, 1024, 4096, 128, 3.0, 2),
    Workload("cfg4_bf16_8x4096x8192_g64_b3.25", BF16, 8, 4096, 8192, 64, 3.25, 3),
    Workload("cfg5_bf16_16x2048x5120_g32_b4.0", BF16, 16, 2048, 5120, 32, 4.0, 4),
)


def f32_to_bf16_bits(x):
    """Round-to-nearest-even narrowing of a finite fp32 array to bf16 bit patterns."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _finish(w, x):
    x = np.ascontiguousarray(x, np.float32)
    return x if w.dtype == F32 else f32_to_bf16_bits(x)


def _cfg1(w, rng):
    ch = rng.choice(w.hidden, size=4, replace=False)
    for _ in range(w.batch):
        x = rng.standard_normal((w.seq, w.hidden), dtype=np.float32)
        x[:, ch] *= np.float32(20.0)
        yield x


def _cfg2(w, rng):
    nch = max(1, w.hidden // 100)
    ch = rng.choice(w.hidden, size=nch, replace=False)
    gain = rng.uniform(10.0, 50.0, size=nch).astype(np.float32)
    for _ in range(w.batch):
        x = rng.standard_normal((w.seq, w.hidden), dtype=np.float32)
        x[:, ch] *= gain[None, :]
        tok = rng.lognormal(0.0, 0.5, size=w.seq).astype(np.float32)
        x *= tok[:, None]
        yield x


def _cfg3(w, rng):
    ch = rng.choice(w.hidden, size=16, replace=False)
    for _ in range(w.batch):
        x = rng.standard_t(3.0, size=(w.seq, w.hidden)).astype(np.float32)
        x[:, ch] *= np.float32(30.0)
        yield x


def _cfg4(w, rng):
    ch = rng.choice(w.hidden, size=32, replace=False)
    for _ in range(w.batch):
        x = rng.standard_normal((w.seq, w.hidden), dtype=np.float32)
        wide = np.nonzero(rng.random(w.seq) < 0.05)[0]
        if wide.size:
            x[wide] = rng.uniform(-8.0, 8.0, size=(wide.size, w.hidden)).astype(np.float32)
        x[:, ch] *= np.float32(40.0)
        yield x


def _cfg5(w, rng):
    for _ in range(w.batch):
        x = rng.standard_normal((w.seq, w.hidden), dtype=np.float32)
        x *= np.float32(1e-3)
        spikes = rng.random((w.seq, w.hidden), dtype=np.float32) < np.float32(0.001)
        x[spikes] *= np.float32(1000.0)
        dead = rng.random(w.seq) < 0.2
        x[dead] = np.float32(0.0)
        yield x


_RECIPES = (_cfg1, _cfg2, _cfg3, _cfg4, _cfg5)


def generate(index, batch=None, seq=None, hidden=None):
    """Tensor of configuration `index` (1-based), optionally with fewer samples / tokens, or with the
    configuration's recipe applied to another hidden size (the name then says so).

    Returns (workload, array): array is float32 [B,S,C] or uint16 (bf16 bits) [B,S,C]."""
    base = CONFIGS[index - 1]
    w = base.with_shape(batch, seq)
    if hidden is not None and hidden != base.hidden:
        w = Workload(f"{base.name}_recipe_at_{w.batch}x{w.seq}x{hidden}", w.dtype, w.batch, w.seq, hidden, w.tile,
                     w.budget_bits, w.seed)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    out = np.empty((w.batch, w.seq, w.hidden), np.float32 if w.dtype == F32 else np.uint16)
    for i, x in enumerate(_RECIPES[index - 1](w, rng)):
        out[i] = _finish(w, x)
    return w, out


def edge_tiles(G, seed=1234):
    """A [n, G] fp32 block of degenerate and adversarial tiles for edge-case tests:
    all-zero, constant, one-hot (each position class), two equal maxima, negative zero,
    subnormals, tied entropies (permutations of one tile), huge and tiny magnitudes."""
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = []
    rows.append(np.zeros(G, np.float32))
    rows.append(np.full(G, 3.25, np.float32))
    rows.append(np.full(G, -0.5, np.float32))
    for d in (0, 1, G // 2, G - 1):
        t = np.zeros(G, np.float32); t[d] = 16.0; rows.append(t)
        t = np.zeros(G, np.float32); t[d] = -7.5; rows.append(t)
    t = rng.standard_normal(G).astype(np.float32); t[3] = 9.0; t[G - 2] = -9.0; rows.append(t)   # equal maxima
    t = rng.standard_normal(G).astype(np.float32); t[5] = 100.0; rows.append(t)                  # clear outlier
    t = np.zeros(G, np.float32); t[::2] = -0.0; t[1] = 1.0; rows.append(t)                        # -0 entries
    t = np.full(G, 1e-40, np.float32); t[7] = -3e-39; rows.append(t)                              # subnormals
    t = rng.standard_normal(G).astype(np.float32) * np.float32(1e-6); rows.append(t)
    t = rng.standard_normal(G).astype(np.float32) * np.float32(3e3); rows.append(t)
    t = rng.standard_normal(G).astype(np.float32) * np.float32(1e5); rows.append(t)              # beyond fp16 range
    base = rng.standard_normal(G).astype(np.float32)
    for _ in range(6):                                                                             # same multiset
        rows.append(base.copy())
    rows.append(base[::-1].copy())
    t = np.arange(G, dtype=np.float32) - G / 2; rows.append(t)
    t = np.ones(G, np.float32); t[G // 2:] = -1.0; rows.append(t)                                 # a Hadamard row
    for _ in range(8):
        rows.append(rng.standard_normal(G).astype(np.float32))
    return np.stack(rows)
