"""tahq: TAH-Quant stage-boundary activation codec for MI355X (gfx950).

The work is done by hand-written HIP kernels in libtahq.so behind a C ABI
(include/tahq.h; include/tahq_naive.h for the backward-pass fixed-point compressor).  This package is argument marshalling only: it hands device
pointers of torch tensors and the current HIP stream to the library.  There is
no CPU or PyTorch fallback: if the library is missing, importing the binding's
functions raises.
"""
from .binding import (  # noqa: F401
    F32, BF16, TahqError, make_config, tahq_config,
    tahq_config_default, tahq_k_per_unit, tahq_packed_size, tahq_workspace_size,
    tahq_encode, tahq_encode_phases, tahq_decode, tahq_encode_noalloc, NOALLOC_MAX_WORKSPACE,
    tahq_samples_packed_size, tahq_samples_workspace_size, tahq_encode_samples, tahq_decode_samples,
    PHASE_PROLOGUE, PHASE_ENTROPY, PHASE_SELECT, PHASE_QUANT, PHASE_ALL, SELECT_MULTI_LAUNCH,
    tahq_tile_entropy, tahq_alloc_tile_entropy, tahq_parse_header,
    tahq_status_string, tahq_version, library_path, Codec,
    tahq_naive_config, make_naive_config, tahq_naive_config_default, tahq_naive_packed_size,
    tahq_naive_encode, tahq_naive_decode,
)
