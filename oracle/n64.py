"""Independent NumPy statement of the backward fixed-point compressor, for pinning the C oracle.
TEST INFRASTRUCTURE ONLY.  Codes by the float64 definition; the stream parsed with unpackbits."""
import numpy as np


def code_range(bits):
    return -(1 << (bits - 1)), (1 << (bits - 1)) - 1


def codes(y, bits):
    """clamp(round-half-even(y)) for already scaled values y (float64); NaN takes the lower bound."""
    lo, hi = code_range(bits)
    y = np.asarray(y, np.float64)
    with np.errstate(invalid="ignore"):
        q = np.clip(np.rint(y), lo, hi)
    return np.where(np.isnan(y), lo, q).astype(np.int64)


def parse_stream(packed, n, bits):
    """Header words and the n signed codes of the payload (LSB-first bit string, two's complement)."""
    packed = np.asarray(packed, np.uint8)
    assert packed.size == 64 + n * bits // 8
    hdr = packed[:64].view("<u4")
    field_bits = np.unpackbits(packed[64:], bitorder="little").reshape(n, bits).astype(np.int64)
    field = (field_bits << np.arange(bits)[None, :]).sum(axis=1)
    q = np.where(field >= (1 << (bits - 1)), field - (1 << bits), field)
    return hdr, q


def values(q, scale):
    """q * fp32(1/c), rounded once to fp32 (the float64 product of a small integer and an fp32 is exact)."""
    rc = np.float32(1.0) / np.float32(scale)
    return (np.asarray(q, np.float64) * np.float64(rc)).astype(np.float32)
