"""ctypes access to the plain-C oracle (oracle/tahq_oracle.c).  TEST INFRASTRUCTURE ONLY.

All arrays are host NumPy arrays.  bf16 tensors travel as uint16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build_oracle

F32, BF16 = 0, 1


class Cfg(C.Structure):
    _fields_ = [
        ("batch", C.c_uint32), ("seq", C.c_uint32), ("hidden", C.c_uint32), ("tile", C.c_uint32),
        ("dtype", C.c_uint32), ("scope", C.c_uint32),
        ("budget_bits", C.c_float), ("tau", C.c_float),
        ("eps_l1", C.c_float), ("eps_log", C.c_float), ("eps_ratio", C.c_float),
        ("alloc_tile", C.c_uint32), ("low_bits", C.c_uint32),
    ]


def make_cfg(batch, seq, hidden, tile, dtype, budget_bits, tau=2.0, eps_l1=1e-8, eps_log=1e-8,
             eps_ratio=1e-8, scope=0, alloc_tile=0, low_bits=0):
    return Cfg(batch, seq, hidden, tile, dtype, scope, budget_bits, tau, eps_l1, eps_log, eps_ratio, alloc_tile,
               low_bits)


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.LIB
        if not os.path.exists(path):
            build_oracle.build()
        L = C.CDLL(path)
        P = C.POINTER
        L.tahq_oracle_k.restype = C.c_uint64
        L.tahq_oracle_k.argtypes = [P(Cfg)]
        L.tahq_oracle_packed_size.restype = C.c_uint64
        L.tahq_oracle_packed_size.argtypes = [P(Cfg)]
        L.tahq_oracle_bf16_rne.restype = C.c_uint16
        L.tahq_oracle_bf16_rne.argtypes = [C.c_float]
        L.tahq_oracle_fp16_widen.restype = C.c_float
        L.tahq_oracle_fp16_widen.argtypes = [C.c_uint16]
        for name in ("tahq_oracle_fp16_rne", "tahq_oracle_fp16_down", "tahq_oracle_fp16_up"):
            getattr(L, name).restype = C.c_uint16
            getattr(L, name).argtypes = [C.c_float]
        L.tahq_oracle_log.restype = C.c_float
        L.tahq_oracle_log.argtypes = [C.c_float]
        L.tahq_oracle_entropy.restype = C.c_float
        L.tahq_oracle_entropy.argtypes = [C.c_void_p, C.c_uint32, C.c_float, C.c_float]
        L.tahq_oracle_entropy_alloc.restype = C.c_float
        L.tahq_oracle_entropy_alloc.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_float, C.c_float]
        L.tahq_oracle_alloc_entropies.restype = C.c_int
        L.tahq_oracle_alloc_entropies.argtypes = [P(Cfg), C.c_void_p, C.c_void_p]
        L.tahq_oracle_outlier.restype = C.c_int
        L.tahq_oracle_outlier.argtypes = [C.c_void_p, C.c_uint32, C.c_float, C.c_float, P(C.c_uint32)]
        L.tahq_oracle_butterfly.restype = None
        L.tahq_oracle_butterfly.argtypes = [C.c_void_p, C.c_uint32]
        for name in ("tahq_oracle_forward_transform", "tahq_oracle_inverse_transform"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [C.c_void_p, C.c_uint32, C.c_uint32]
        L.tahq_oracle_quant_params.restype = None
        L.tahq_oracle_quant_params.argtypes = [C.c_float, C.c_float, C.c_uint32, P(C.c_uint16), P(C.c_uint16)]
        L.tahq_oracle_quant_code.restype = C.c_uint32
        L.tahq_oracle_quant_code.argtypes = [C.c_float, C.c_uint16, C.c_uint16, C.c_uint32]
        L.tahq_oracle_dequant.restype = C.c_float
        L.tahq_oracle_dequant.argtypes = [C.c_uint32, C.c_uint16, C.c_uint16]
        L.tahq_oracle_allocate.restype = C.c_int
        L.tahq_oracle_allocate.argtypes = [P(Cfg), C.c_void_p, C.c_void_p]
        L.tahq_oracle_tile_stats.restype = C.c_int
        L.tahq_oracle_tile_stats.argtypes = [P(Cfg), C.c_void_p] + [C.c_void_p] * 4
        L.tahq_oracle_encode.restype = C.c_int
        L.tahq_oracle_encode.argtypes = [P(Cfg), C.c_void_p, C.c_void_p, C.c_uint64]
        L.tahq_oracle_decode.restype = C.c_int
        L.tahq_oracle_decode.argtypes = [P(Cfg), C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _check_input(cfg, x):
    want = np.float32 if cfg.dtype == F32 else np.uint16
    assert x.dtype == want and x.flags.c_contiguous, (x.dtype, want)
    assert x.size == cfg.batch * cfg.seq * cfg.hidden


def n_tiles(cfg):
    return cfg.batch * cfg.seq * (cfg.hidden // cfg.tile)


def low_bits(cfg):
    return cfg.low_bits or 3


def tiles_per_alloc(cfg):
    return cfg.alloc_tile // cfg.tile if cfg.alloc_tile else 1


def alloc_entropies(cfg, x):
    """Entropy of every allocation tile (one per quantization tile when A = G)."""
    _check_input(cfg, x)
    H = np.empty(n_tiles(cfg) // tiles_per_alloc(cfg), np.float32)
    rc = lib().tahq_oracle_alloc_entropies(C.byref(cfg), _ptr(x), _ptr(H))
    assert rc == 0, rc
    return H


def k_per_unit(cfg):
    return int(lib().tahq_oracle_k(C.byref(cfg)))


def packed_size(cfg):
    return int(lib().tahq_oracle_packed_size(C.byref(cfg)))


def tile_stats(cfg, x):
    """Entropy, pivot byte, min and max (of the domain that is quantized) of every tile."""
    _check_input(cfg, x)
    T = n_tiles(cfg)
    H = np.empty(T, np.float32)
    pivot = np.empty(T, np.uint8)
    mn = np.empty(T, np.float32)
    mx = np.empty(T, np.float32)
    rc = lib().tahq_oracle_tile_stats(C.byref(cfg), _ptr(x), _ptr(H), _ptr(pivot), _ptr(mn), _ptr(mx))
    assert rc == 0, rc
    return H, pivot, mn, mx


def allocate(cfg, H):
    """H: one entropy per allocation tile; returns the width (lo or lo+1) of every quantization tile."""
    H = np.ascontiguousarray(H, np.float32)
    assert H.size == n_tiles(cfg) // tiles_per_alloc(cfg)
    width = np.empty(n_tiles(cfg), np.uint8)
    rc = lib().tahq_oracle_allocate(C.byref(cfg), _ptr(H), _ptr(width))
    assert rc == 0, rc
    return width


def encode(cfg, x):
    _check_input(cfg, x)
    size = packed_size(cfg)
    assert size > 0, "invalid configuration"
    out = np.empty(size, np.uint8)
    rc = lib().tahq_oracle_encode(C.byref(cfg), _ptr(x), _ptr(out), size)
    assert rc == 0, rc
    return out


def decode(cfg, packed, out_dtype=F32):
    packed = np.ascontiguousarray(packed, np.uint8)
    n = cfg.batch * cfg.seq * cfg.hidden
    out = np.empty(n, np.float32 if out_dtype == F32 else np.uint16)
    rc = lib().tahq_oracle_decode(C.byref(cfg), _ptr(packed), packed.size, _ptr(out), out_dtype)
    assert rc == 0, rc
    return out


# --- scalar / per-tile helpers, exposed for the pin tests -------------------

def log(u):
    return float(lib().tahq_oracle_log(np.float32(u)))


def fp16_widen(h):
    return float(lib().tahq_oracle_fp16_widen(int(h)))


def fp16_rne(x):
    return int(lib().tahq_oracle_fp16_rne(np.float32(x)))


def fp16_down(x):
    return int(lib().tahq_oracle_fp16_down(np.float32(x)))


def fp16_up(x):
    return int(lib().tahq_oracle_fp16_up(np.float32(x)))


def bf16_rne(x):
    return int(lib().tahq_oracle_bf16_rne(np.float32(x)))


def entropy(v, eps_l1=1e-8, eps_log=1e-8):
    v = np.ascontiguousarray(v, np.float32)
    return float(lib().tahq_oracle_entropy(_ptr(v), v.size, eps_l1, eps_log))


def entropy_alloc(v, G, eps_l1=1e-8, eps_log=1e-8):
    """Entropy of one allocation tile v of m*G channels."""
    v = np.ascontiguousarray(v, np.float32)
    assert v.size % G == 0
    return float(lib().tahq_oracle_entropy_alloc(_ptr(v), G, v.size // G, eps_l1, eps_log))


def outlier(v, tau=2.0, eps_ratio=1e-8):
    v = np.ascontiguousarray(v, np.float32)
    d = C.c_uint32(0)
    flag = lib().tahq_oracle_outlier(_ptr(v), v.size, tau, eps_ratio, C.byref(d))
    return bool(flag), int(d.value)


def butterfly(v):
    v = np.array(v, np.float32, copy=True)
    lib().tahq_oracle_butterfly(_ptr(v), v.size)
    return v


def forward_transform(v, d):
    v = np.array(v, np.float32, copy=True)
    lib().tahq_oracle_forward_transform(_ptr(v), v.size, d)
    return v


def inverse_transform(v, d):
    v = np.array(v, np.float32, copy=True)
    lib().tahq_oracle_inverse_transform(_ptr(v), v.size, d)
    return v


def quant_params(mn, mx, b):
    s, z = C.c_uint16(0), C.c_uint16(0)
    lib().tahq_oracle_quant_params(np.float32(mn), np.float32(mx), b, C.byref(s), C.byref(z))
    return int(s.value), int(z.value)


def quant_code(y, s16, z16, b):
    return int(lib().tahq_oracle_quant_code(np.float32(y), s16, z16, b))


def dequant(q, s16, z16):
    return float(lib().tahq_oracle_dequant(q, s16, z16))
