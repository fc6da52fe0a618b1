"""ctypes binding of libtahq.so: same names as the C ABI, marshalling only."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
# TAHQ_LIBRARY lets an experiment load another build of the same library
_LIB_PATH = os.environ.get("TAHQ_LIBRARY") or os.path.join(HERE, "libtahq.so")

F32, BF16 = 0, 1


class TahqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {tahq_status_string(status)} (status {status})")


class tahq_config(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("batch", C.c_uint32), ("seq", C.c_uint32), ("hidden", C.c_uint32),
        ("tile", C.c_uint32), ("dtype", C.c_uint32), ("scope", C.c_uint32),
        ("budget_bits", C.c_float), ("tau", C.c_float),
        ("eps_l1", C.c_float), ("eps_log", C.c_float), ("eps_ratio", C.c_float),
        ("alloc_tile", C.c_uint32), ("low_bits", C.c_uint32),
    ]


class tahq_naive_config(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("batch", C.c_uint32), ("seq", C.c_uint32), ("hidden", C.c_uint32),
        ("dtype", C.c_uint32), ("bits", C.c_uint32), ("scale", C.c_float),
    ]


_lib = None


def library_path():
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2506_01352_amd.build` "
            "(there is no fallback path)")
    L = C.CDLL(_LIB_PATH)
    P = C.POINTER(tahq_config)
    L.tahq_config_default.restype = None
    L.tahq_config_default.argtypes = [P]
    L.tahq_k_per_unit.restype = C.c_uint64
    L.tahq_k_per_unit.argtypes = [P]
    L.tahq_packed_size.restype = C.c_size_t
    L.tahq_packed_size.argtypes = [P]
    L.tahq_workspace_size.restype = C.c_size_t
    L.tahq_workspace_size.argtypes = [P]
    L.tahq_encode.restype = C.c_int
    L.tahq_encode.argtypes = [P, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tahq_encode_noalloc.restype = C.c_int
    L.tahq_encode_noalloc.argtypes = [P, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tahq_encode_phases.restype = C.c_int
    L.tahq_encode_phases.argtypes = [P, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_uint32,
                                     C.c_void_p]
    L.tahq_samples_packed_size.restype = C.c_size_t
    L.tahq_samples_packed_size.argtypes = [P, C.c_uint32]
    L.tahq_samples_workspace_size.restype = C.c_size_t
    L.tahq_samples_workspace_size.argtypes = [P, C.c_uint32]
    L.tahq_encode_samples.restype = C.c_int
    L.tahq_encode_samples.argtypes = [P, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p,
                                      C.c_size_t, C.c_void_p]
    L.tahq_decode_samples.restype = C.c_int
    L.tahq_decode_samples.argtypes = [P, C.c_uint32, C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p, C.c_uint32,
                                      C.c_void_p]
    L.tahq_decode.restype = C.c_int
    L.tahq_decode.argtypes = [P, C.c_void_p, C.c_size_t, C.c_void_p, C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tahq_tile_entropy.restype = C.c_int
    L.tahq_tile_entropy.argtypes = [P, C.c_void_p, C.c_void_p, C.c_void_p]
    L.tahq_alloc_tile_entropy.restype = C.c_int
    L.tahq_alloc_tile_entropy.argtypes = [P, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tahq_parse_header.restype = C.c_int
    L.tahq_parse_header.argtypes = [C.c_void_p, P]
    L.tahq_status_string.restype = C.c_char_p
    L.tahq_status_string.argtypes = [C.c_int]
    L.tahq_version.restype = C.c_uint32
    L.tahq_version.argtypes = []
    PN = C.POINTER(tahq_naive_config)
    L.tahq_naive_config_default.restype = None
    L.tahq_naive_config_default.argtypes = [PN]
    L.tahq_naive_packed_size.restype = C.c_size_t
    L.tahq_naive_packed_size.argtypes = [PN]
    L.tahq_naive_encode.restype = C.c_int
    L.tahq_naive_encode.argtypes = [PN, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tahq_naive_decode.restype = C.c_int
    L.tahq_naive_decode.argtypes = [PN, C.c_void_p, C.c_size_t, C.c_void_p, C.c_uint32, C.c_void_p]
    _lib = L
    return L


def tahq_config_default():
    cfg = tahq_config()
    _load().tahq_config_default(C.byref(cfg))
    return cfg


def make_config(batch, seq, hidden, tile, dtype, budget_bits, tau=2.0, eps_l1=1e-8, eps_log=1e-8,
                eps_ratio=1e-8, scope=0, alloc_tile=0, low_bits=0):
    cfg = tahq_config_default()
    cfg.alloc_tile = alloc_tile
    cfg.low_bits = low_bits
    cfg.batch, cfg.seq, cfg.hidden, cfg.tile = batch, seq, hidden, tile
    cfg.dtype, cfg.scope = dtype, scope
    cfg.budget_bits, cfg.tau = budget_bits, tau
    cfg.eps_l1, cfg.eps_log, cfg.eps_ratio = eps_l1, eps_log, eps_ratio
    return cfg


def tahq_k_per_unit(cfg):
    return int(_load().tahq_k_per_unit(C.byref(cfg)))


def tahq_packed_size(cfg):
    return int(_load().tahq_packed_size(C.byref(cfg)))


def tahq_workspace_size(cfg):
    return int(_load().tahq_workspace_size(C.byref(cfg)))


def tahq_status_string(status):
    return _load().tahq_status_string(int(status)).decode()


def tahq_version():
    return int(_load().tahq_version())


def _dev_ptr(t):
    """Device address of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    assert t.is_cuda and t.is_contiguous(), "device tensor, contiguous"
    return C.c_void_p(t.data_ptr())


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


_ESIZE = {F32: 4, BF16: 2}


def _check_tensor(where, name, t, elements, dtype):
    """The C ABI carries no capacity for the activation tensors: refuse, on the host, a tensor that is shorter than
    batch*seq*hidden elements of `dtype`, or whose elements have another size (byte buffers are taken as they are)."""
    if t is None or isinstance(t, int):
        return
    esize = _ESIZE.get(dtype)
    if esize is None:
        return                                   # the library rejects the dtype itself
    if t.element_size() not in (1, esize):
        raise ValueError(f"{where}: {name} has {t.element_size()}-byte elements, the configuration says {esize}")
    if _nbytes(t) < elements * esize:
        raise ValueError(f"{where}: {name} holds {_nbytes(t)} bytes, the configuration needs {elements * esize}")


def _elements(cfg):
    return cfg.batch * cfg.seq * cfg.hidden


def _stream_handle(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def tahq_encode(cfg, d_in, d_packed, d_workspace, stream=None, packed_capacity=None, workspace_capacity=None):
    """Enqueue the encoder.  All tensors are device tensors owned by the caller."""
    cap = _nbytes(d_packed) if packed_capacity is None else packed_capacity
    wcap = _nbytes(d_workspace) if workspace_capacity is None else workspace_capacity
    _check_tensor("tahq_encode", "d_in", d_in, _elements(cfg), cfg.dtype)
    rc = _load().tahq_encode(C.byref(cfg), _dev_ptr(d_in), _dev_ptr(d_packed), cap, _dev_ptr(d_workspace), wcap,
                             _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_encode")


NOALLOC_MAX_WORKSPACE = 32 << 20     # TAHQ_NOALLOC_MAX_WORKSPACE of include/tahq.h


def tahq_encode_noalloc(cfg, d_in, d_packed, stream=None, packed_capacity=None):
    """tahq_encode on the library's built-in scratch: no workspace argument, nothing allocated."""
    cap = _nbytes(d_packed) if packed_capacity is None else packed_capacity
    _check_tensor("tahq_encode_noalloc", "d_in", d_in, _elements(cfg), cfg.dtype)
    rc = _load().tahq_encode_noalloc(C.byref(cfg), _dev_ptr(d_in), _dev_ptr(d_packed), cap, _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_encode_noalloc")


PHASE_PROLOGUE, PHASE_ENTROPY, PHASE_SELECT, PHASE_QUANT, PHASE_ALL = 1, 2, 4, 8, 15
SELECT_MULTI_LAUNCH = 16      # option bit for tahq_encode_phases: see include/tahq.h


def tahq_encode_phases(cfg, d_in, d_packed, d_workspace, phases, stream=None):
    _check_tensor("tahq_encode_phases", "d_in", d_in, _elements(cfg), cfg.dtype)
    rc = _load().tahq_encode_phases(C.byref(cfg), _dev_ptr(d_in), _dev_ptr(d_packed), _nbytes(d_packed),
                                    _dev_ptr(d_workspace), _nbytes(d_workspace), phases, _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_encode_phases")


def tahq_decode(cfg, d_packed, d_out, out_dtype, stream=None, packed_bytes=None):
    nbytes = _nbytes(d_packed) if packed_bytes is None else packed_bytes
    _check_tensor("tahq_decode", "d_out", d_out, _elements(cfg), out_dtype)
    rc = _load().tahq_decode(C.byref(cfg), _dev_ptr(d_packed), nbytes, _dev_ptr(d_out), out_dtype, None, 0,
                             _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_decode")


def tahq_samples_packed_size(cfg, count):
    return int(_load().tahq_samples_packed_size(C.byref(cfg), count))


def tahq_samples_workspace_size(cfg, count):
    return int(_load().tahq_samples_workspace_size(C.byref(cfg), count))


def tahq_encode_samples(cfg, first, count, d_in, d_packed, d_workspace, stream=None):
    """Samples [first, first + count) of the whole tensor d_in -> a self-contained stream in d_packed."""
    _check_tensor("tahq_encode_samples", "d_in", d_in, _elements(cfg), cfg.dtype)
    rc = _load().tahq_encode_samples(C.byref(cfg), first, count, _dev_ptr(d_in), _dev_ptr(d_packed), _nbytes(d_packed),
                                     _dev_ptr(d_workspace), _nbytes(d_workspace), _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_encode_samples")


def tahq_decode_samples(cfg, first, count, d_packed, d_out, out_dtype, stream=None):
    """A stream of tahq_encode_samples -> samples [first, first + count) of the whole tensor d_out."""
    _check_tensor("tahq_decode_samples", "d_out", d_out, _elements(cfg), out_dtype)
    rc = _load().tahq_decode_samples(C.byref(cfg), first, count, _dev_ptr(d_packed), _nbytes(d_packed), _dev_ptr(d_out),
                                     out_dtype, _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_decode_samples")


def tahq_tile_entropy(cfg, d_in, d_entropy, stream=None):
    _check_tensor("tahq_tile_entropy", "d_in", d_in, _elements(cfg), cfg.dtype)
    _check_tensor("tahq_tile_entropy", "d_entropy", d_entropy, _elements(cfg) // max(cfg.tile, 1), F32)
    rc = _load().tahq_tile_entropy(C.byref(cfg), _dev_ptr(d_in), _dev_ptr(d_entropy), _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_tile_entropy")


def tahq_alloc_tile_entropy(cfg, d_in, d_entropy, d_workspace, stream=None):
    _check_tensor("tahq_alloc_tile_entropy", "d_in", d_in, _elements(cfg), cfg.dtype)
    _check_tensor("tahq_alloc_tile_entropy", "d_entropy", d_entropy,
                  _elements(cfg) // max(cfg.alloc_tile or cfg.tile, 1), F32)
    rc = _load().tahq_alloc_tile_entropy(C.byref(cfg), _dev_ptr(d_in), _dev_ptr(d_entropy), _dev_ptr(d_workspace),
                                         _nbytes(d_workspace), _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_alloc_tile_entropy")


def tahq_parse_header(header_bytes):
    buf = C.create_string_buffer(bytes(header_bytes[:64]), 64)
    cfg = tahq_config()
    rc = _load().tahq_parse_header(buf, C.byref(cfg))
    if rc != 0:
        raise TahqError(rc, "tahq_parse_header")
    return cfg


# ---- backward-pass fixed-point compressor (include/tahq_naive.h)

def tahq_naive_config_default():
    cfg = tahq_naive_config()
    _load().tahq_naive_config_default(C.byref(cfg))
    return cfg


def make_naive_config(batch, seq, hidden, dtype, bits, scale=1.0):
    cfg = tahq_naive_config_default()
    cfg.batch, cfg.seq, cfg.hidden, cfg.dtype, cfg.bits, cfg.scale = batch, seq, hidden, dtype, bits, scale
    return cfg


def tahq_naive_packed_size(cfg):
    return int(_load().tahq_naive_packed_size(C.byref(cfg)))


def tahq_naive_encode(cfg, d_in, d_packed, stream=None, packed_capacity=None):
    cap = _nbytes(d_packed) if packed_capacity is None else packed_capacity
    _check_tensor("tahq_naive_encode", "d_in", d_in, _elements(cfg), cfg.dtype)
    rc = _load().tahq_naive_encode(C.byref(cfg), _dev_ptr(d_in), _dev_ptr(d_packed), cap, _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_naive_encode")


def tahq_naive_decode(cfg, d_packed, d_out, out_dtype, stream=None, packed_bytes=None):
    nbytes = _nbytes(d_packed) if packed_bytes is None else packed_bytes
    _check_tensor("tahq_naive_decode", "d_out", d_out, _elements(cfg), out_dtype)
    rc = _load().tahq_naive_decode(C.byref(cfg), _dev_ptr(d_packed), nbytes, _dev_ptr(d_out), out_dtype,
                                   _stream_handle(stream))
    if rc != 0:
        raise TahqError(rc, "tahq_naive_decode")


class Codec:
    """Buffers for one configuration, allocated once through torch, and the two calls on them."""

    def __init__(self, cfg, device="cuda:0", out_dtype=None):
        import torch
        self.cfg = cfg
        self.out_dtype = cfg.dtype if out_dtype is None else out_dtype
        size = tahq_packed_size(cfg)
        if size == 0:
            raise TahqError(2, "tahq_packed_size")
        n = cfg.batch * cfg.seq * cfg.hidden
        self.packed = torch.empty(size, dtype=torch.uint8, device=device)
        self.workspace = torch.empty(max(tahq_workspace_size(cfg), 16), dtype=torch.uint8, device=device)
        self.out = torch.empty(n, dtype=torch.float32 if self.out_dtype == F32 else torch.bfloat16, device=device)

    def encode(self, d_in, stream=None):
        tahq_encode(self.cfg, d_in, self.packed, self.workspace, stream)
        return self.packed

    def decode(self, stream=None):
        tahq_decode(self.cfg, self.packed, self.out, self.out_dtype, stream)
        return self.out
