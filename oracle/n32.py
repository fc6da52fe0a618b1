"""ctypes access to the plain-C oracle of the backward fixed-point compressor (oracle/naive_oracle.c).
TEST INFRASTRUCTURE ONLY.  Host NumPy arrays; bf16 tensors travel as uint16 bit patterns."""
import ctypes as C
import os

import numpy as np

from . import build_oracle

F32, BF16 = 0, 1


class Cfg(C.Structure):
    _fields_ = [("batch", C.c_uint32), ("seq", C.c_uint32), ("hidden", C.c_uint32), ("dtype", C.c_uint32),
                ("bits", C.c_uint32), ("scale", C.c_float)]


def make_cfg(batch, seq, hidden, dtype, bits, scale=1.0):
    return Cfg(batch, seq, hidden, dtype, bits, scale)


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.NAIVE_LIB
        if not os.path.exists(path):
            build_oracle.build()
        L = C.CDLL(path)
        P = C.POINTER(Cfg)
        L.naive_oracle_packed_size.restype = C.c_uint64
        L.naive_oracle_packed_size.argtypes = [P]
        L.naive_oracle_code.restype = C.c_int32
        L.naive_oracle_code.argtypes = [C.c_float, C.c_float, C.c_uint32]
        L.naive_oracle_value.restype = C.c_float
        L.naive_oracle_value.argtypes = [C.c_int32, C.c_float]
        L.naive_oracle_encode.restype = C.c_int
        L.naive_oracle_encode.argtypes = [P, C.c_void_p, C.c_void_p, C.c_uint64]
        L.naive_oracle_decode.restype = C.c_int
        L.naive_oracle_decode.argtypes = [P, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def packed_size(cfg):
    return int(lib().naive_oracle_packed_size(C.byref(cfg)))


def code(g, scale, bits):
    return int(lib().naive_oracle_code(np.float32(g), np.float32(scale), bits))


def value(q, scale):
    return float(lib().naive_oracle_value(int(q), np.float32(scale)))


def encode(cfg, x):
    want = np.float32 if cfg.dtype == F32 else np.uint16
    assert x.dtype == want and x.flags.c_contiguous and x.size == cfg.batch * cfg.seq * cfg.hidden
    size = packed_size(cfg)
    assert size > 0, "invalid configuration"
    out = np.empty(size, np.uint8)
    rc = lib().naive_oracle_encode(C.byref(cfg), _ptr(x), _ptr(out), size)
    assert rc == 0, rc
    return out


def decode(cfg, packed, out_dtype=F32):
    packed = np.ascontiguousarray(packed, np.uint8)
    out = np.empty(cfg.batch * cfg.seq * cfg.hidden, np.float32 if out_dtype == F32 else np.uint16)
    rc = lib().naive_oracle_decode(C.byref(cfg), _ptr(packed), packed.size, _ptr(out), out_dtype)
    assert rc == 0, rc
    return out
