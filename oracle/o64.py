"""Float64 NumPy transcription of the paper's equations.  TEST INFRASTRUCTURE ONLY.

This is the mathematics with library routines (np.log, a dense Sylvester matrix
from scipy, np.lexsort, np.float16, np.unpackbits): no operation order, no fast
transform, no hand-written bit tricks.  The fp32 C oracle is pinned against it,
and the byte stream the C oracle writes is parsed and decoded here independently.

Sections cited: Sec. 3.1 (tiles), Sec. 3.2 Eq. 1-2 (entropy) and top-p% selection,
Sec. 3.3 Eq. 3-4 (outlier test, pivot swap, Hadamard), Sec. 3.4 (byte stream),
Alg. 1 step 5 (dequantize).
"""
import numpy as np
from scipy.linalg import hadamard


def tiles_of(x, G):
    """Sec. 3.1: [B,S,C] -> [T,G], contiguous channels of a token form a tile."""
    return np.asarray(x, np.float64).reshape(-1, G)


def entropy(tiles, eps_l1=1e-8, eps_log=1e-8):
    """Eq. 1-2 with the Shannon sign (H high for evenly spread energy)."""
    a = np.abs(np.asarray(tiles, np.float64))
    p = a / (a.sum(axis=-1, keepdims=True) + eps_l1)
    return -(p * np.log(p + eps_log)).sum(axis=-1)


def outlier(tiles, tau=2.0, eps_ratio=1e-8):
    """Eq. 3: (flag, d) per tile; d = first index of the largest magnitude."""
    a = np.abs(np.asarray(tiles, np.float64))
    d = a.argmax(axis=-1)
    srt = np.sort(a, axis=-1)
    a1, a2 = srt[..., -1], srt[..., -2]
    with np.errstate(invalid="ignore"):
        flag = a1 > tau * (a2 + eps_ratio)
    return flag, d


def sylvester(G):
    """H_G in {+1,-1}^{GxG}, natural (Sylvester) order: H[i,j] = (-1)^popcount(i&j)."""
    return hadamard(G).astype(np.float64)


def swap_matrix(G, d):
    """P_d: the permutation matrix that swaps coordinates 1 and d (0-based: 0 and d)."""
    P = np.eye(G)
    P[[0, d]] = P[[d, 0]]
    return P


def forward_transform(tile, d):
    """Eq. 4: alpha P_d (1/sqrt(G)) H_G, as dense matrix products."""
    G = len(tile)
    return np.asarray(tile, np.float64) @ swap_matrix(G, d) @ sylvester(G) / np.sqrt(G)


def inverse_transform(y, d):
    G = len(y)
    return np.asarray(y, np.float64) @ sylvester(G).T / np.sqrt(G) @ swap_matrix(G, d).T


def k_per_unit(n, budget, low=3):
    """Sec. 3.2: top-p% with p = budget - low, rounded to the nearest tile count."""
    return int(min(max(np.floor(float(budget) * n - float(low) * n + 0.5), 0), n))


def allocate(H, n_units, k, low=3):
    """Per ranking unit: the k highest entropies get low+1 bits (ties: lower index), the rest low."""
    H = np.asarray(H).reshape(n_units, -1)
    n = H.shape[1]
    width = np.full(H.shape, low, np.uint8)
    for u in range(n_units):
        order = np.lexsort((np.arange(n), -H[u].astype(np.float64)))
        width[u, order[:k]] = low + 1
    return width.reshape(-1)


# ---- byte stream (Sec. 3.4), parsed with NumPy views only ------------------

def _pad64(x):
    return (x + 63) // 64 * 64


def section_offsets(T, G, n_units, k, low=3):
    off = {}
    off["bitmap"] = 64
    off["ranks"] = off["bitmap"] + _pad64((T + 7) // 8)
    off["pivot"] = off["ranks"] + _pad64(4 * ((T + 63) // 64))
    off["scale"] = off["pivot"] + _pad64(T)
    off["zero"] = off["scale"] + _pad64(2 * T)
    off["payload"] = off["zero"] + _pad64(2 * T)
    off["total"] = off["payload"] + (G // 8) * (low * T + n_units * k)
    return off


def parse_stream(packed, T, G, n_units, k, low=3):
    """Split the stream into its sections; codes come back as a [T,G] uint8 array.  k counts the wide
    (low+1 bit) quantization tiles per ranking unit."""
    packed = np.asarray(packed, np.uint8)
    off = section_offsets(T, G, n_units, k, low)
    assert packed.size >= off["total"]
    hdr = packed[:64]
    bits = np.unpackbits(packed[off["bitmap"]:off["bitmap"] + (T + 7) // 8], bitorder="little")[:T]
    ranks = packed[off["ranks"]:off["ranks"] + 4 * ((T + 63) // 64)].view("<u4")
    pivot = packed[off["pivot"]:off["pivot"] + T]
    scale = packed[off["scale"]:off["scale"] + 2 * T].view("<f2")
    zero = packed[off["zero"]:off["zero"] + 2 * T].view("<f2")
    width = np.where(bits == 1, low + 1, low).astype(np.int64)
    rank_of = np.concatenate([[0], np.cumsum(bits)[:-1]]).astype(np.int64)   # wide tiles before j
    start = off["payload"] + (G // 8) * (low * np.arange(T, dtype=np.int64) + rank_of)
    codes = np.zeros((T, G), np.uint8)
    for b in (low, low + 1):
        sel = np.nonzero(width == b)[0]
        if sel.size == 0:
            continue
        nbytes = G * b // 8
        idx = start[sel, None] + np.arange(nbytes)[None, :]
        tile_bits = np.unpackbits(packed[idx], axis=1, bitorder="little")      # LSB-first bit string
        fields = tile_bits.reshape(sel.size, G, b)
        codes[sel] = (fields * (1 << np.arange(b))[None, None, :]).sum(axis=2)
    return dict(header=hdr, bits=bits, ranks=ranks, pivot=pivot, scale=scale, zero=zero,
                width=width, rank_of=rank_of, codes=codes, offsets=off)


def decode_stream(packed, T, G, n_units, k, low=3):
    """Alg. 1 step 5 in float64: q*s + z, then H^T and P_d for transformed tiles."""
    s = parse_stream(packed, T, G, n_units, k, low)
    y = s["codes"].astype(np.float64) * s["scale"].astype(np.float64)[:, None] \
        + s["zero"].astype(np.float64)[:, None]
    out = y.copy()
    Hm = sylvester(G)
    flagged = np.nonzero(s["pivot"] & 0x80)[0]
    if flagged.size:
        t = y[flagged] @ Hm.T / np.sqrt(G)
        d = (s["pivot"][flagged] & 0x7F).astype(np.int64)
        r = np.arange(flagged.size)
        t0 = t[r, 0].copy()
        t[r, 0] = t[r, d]
        t[r, d] = t0
        out[flagged] = t
    return out, s


def minmax_group_quantize(tiles, b):
    """Textbook asymmetric per-group min-max quantizer in float64 (no metadata rounding):
    q = clip(rint((y - mn)/s), 0, 2^b-1), s = (mx - mn)/(2^b-1); returns (q, s, mn)."""
    y = np.asarray(tiles, np.float64)
    mn = y.min(axis=-1, keepdims=True)
    mx = y.max(axis=-1, keepdims=True)
    L = (1 << b) - 1
    s = (mx - mn) / L
    s = np.where(s == 0, 1.0, s)
    q = np.clip(np.rint((y - mn) / s), 0, L)
    return q, s, mn
