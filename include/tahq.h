/*
 * tahq -- TAH-Quant stage-boundary activation codec for AMD MI355X (gfx950).
 *
 * C ABI of libtahq.so.  The library encodes a contiguous row-major activation
 * tensor [batch, seq, hidden] (fp32 or bf16) into one byte stream of fixed,
 * data-independent size and decodes it back.  Per tile of `tile` contiguous
 * channels of one token it computes (paper sections in brackets):
 *
 *   - the entropy of the tile's normalized magnitudes        [Sec. 3.2, Eq. 1-2]
 *   - the outlier test on the two largest magnitudes          [Sec. 3.3, Eq. 3]
 *   - for outlier tiles, the pivot swap P_d and the Hadamard
 *     transform (1/sqrt(G)) H_G                               [Sec. 3.3, Eq. 4]
 *   - 3- or 4-bit width: the top-p% highest-entropy tiles of
 *     every sample get 4 bits, p = budget_bits - 3            [Sec. 3.2]
 *     (lo and lo+1 bits with p = budget_bits - lo if low_bits
 *     selects another pair of neighbouring widths, e.g. the
 *     INT2/INT3 mix of the appendix on bit allocation)
 *     (entropy and ranking may run on allocation tiles of
 *     A = alloc_tile channels, A a multiple of `tile`; the
 *     quantization tiles inside one share its width)
 *   - asymmetric uniform quantization with a per-tile scale
 *     and zero-point                                          [Sec. 3.1, 3.3]
 *   - packing of codes and metadata into one uint8 stream     [Sec. 3.4]
 *
 * and the decoder inverts every step                          [Alg. 1, step 5].
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers (HIP global memory on the current
 *     device); `cfg` and all other pointers are HOST pointers.
 *   - The caller owns every buffer.  The library allocates nothing and never
 *     synchronizes: it validates on the host, then only enqueues kernels on `stream`.
 *   - Device buffers must be 16-byte aligned and must not overlap.
 *   - Argument errors are returned before anything is enqueued.  Data-dependent
 *     conditions (NaN/Inf inputs, magnitudes beyond the binary16 range of the
 *     metadata, +-65504) are not detected: the result is defined but lossy.
 *   - A failed launch is reported as TAHQ_ERR_HIP, and nothing is enqueued after it.  Every launch's
 *     own status is used: an error that the caller's earlier HIP work left pending in the thread is
 *     neither reported here nor cleared.
 *   - The only thing the library remembers between calls is, per kernel and device, how many
 *     workgroups of the kernel the device holds at once (a query of the runtime on first use; it is
 *     not a stream operation and may happen while a stream is being captured).
 *
 * Stream layout (little-endian; every section padded to 64 bytes), T = number
 * of tiles = batch*seq*hidden/tile, k = wide (lo+1 bit) allocation tiles per ranking unit:
 *   header   64 B   "TAHQ", version, dtype, batch, seq, hidden, tile, scope, k,
 *                   budget, tau, eps_l1, eps_log, eps_ratio, A, lo (32-bit words)
 *   bitmap   T bits         tile j -> byte j>>3, bit j&7; 1 = wide tile (lo+1 bits; 4 by default)
 *   ranks    uint32[ceil(T/64)]   wide tiles before each group of 64 tiles
 *   pivot    uint8[T]       bit 7 = tile was transformed, bits 0..6 = pivot index d
 *   scale    binary16[T]    quantization step (rounded up)
 *   zero     binary16[T]    zero-point = tile minimum (rounded down)
 *   payload  tile j at byte (tile/8)*(lo*j + rank(j)), tile*b/8 bytes; element i
 *            occupies bits [b*i, b*i+b) of the tile's LSB-first bit string
 */
#ifndef TAHQ_H
#define TAHQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Opaque stand-in for hipStream_t so that this header needs no HIP include;
 * pass the hipStream_t value itself (NULL = the default stream). */
typedef void *tahq_stream;

typedef enum {
    TAHQ_OK = 0,
    TAHQ_ERR_NULL = 1,                 /* a required pointer is NULL                     */
    TAHQ_ERR_INVALID_ARG = 2,          /* zero dimension, hidden % tile != 0, alloc_tile not a multiple of tile dividing hidden,
                                          budget outside [3,4] or NaN, bad enum */
    TAHQ_ERR_UNSUPPORTED = 3,          /* tile not in {8, 16, 32, 64, 128}, more than 2^31 tiles, or more than
                                          65535 ranking units of more than 32768 tiles each */
    TAHQ_ERR_BUFFER_TOO_SMALL = 4,     /* packed capacity / packed_bytes below tahq_packed_size */
    TAHQ_ERR_WORKSPACE_TOO_SMALL = 5,  /* workspace capacity below tahq_workspace_size   */
    TAHQ_ERR_MISALIGNED = 6,           /* a device pointer is not 16-byte aligned        */
    TAHQ_ERR_HIP = 7,                  /* a kernel launch failed                         */
    TAHQ_ERR_TOO_LARGE = 8             /* tahq_encode_noalloc: tahq_workspace_size(cfg) exceeds TAHQ_NOALLOC_MAX_WORKSPACE */
} tahq_status;

typedef enum { TAHQ_F32 = 0, TAHQ_BF16 = 1 } tahq_dtype;

typedef struct {
    uint32_t struct_size;   /* = sizeof(tahq_config); set by tahq_config_default.  48 and 52 (callers built
                               before alloc_tile / low_bits existed) are accepted; the missing
                               fields then count as 0                                               */
    uint32_t batch;         /* B                                                                  */
    uint32_t seq;           /* S                                                                  */
    uint32_t hidden;        /* C; tensor is contiguous row-major [B, S, C]                        */
    uint32_t tile;          /* G, the quantization tile: 8, 16, 32, 64 (the paper's default) or 128 */
    uint32_t dtype;         /* tahq_dtype of the activation tensor                                */
    uint32_t scope;         /* 0 = rank the tiles of every sample (the paper); 1 = rank the whole tensor */
    float budget_bits;      /* mean payload bits per element, in [lo, lo+1] = [3.0, 4.0] by default */
    float tau;              /* outlier threshold of Eq. 3; default 2.0; +inf = never transform    */
    float eps_l1;           /* epsilon of Eq. 1;   default 1e-8                                   */
    float eps_log;          /* varsigma of Eq. 2;  default 1e-8                                   */
    float eps_ratio;        /* varrho of Eq. 3;    default 1e-8                                   */
    uint32_t alloc_tile;    /* A, the allocation tile of Sec. 3.2: a multiple of G that divides C;
                               0 = G (the paper's default); A = C is token-level allocation        */
    uint32_t low_bits;      /* lo, 1..7: the two code widths are lo and lo+1 bits and budget_bits lies
                               in [lo, lo+1].  3 (or 0) = INT3/INT4, the paper's setting; 2 = the
                               INT2/INT3 mix of the appendix on bit allocation; any other pair of
                               neighbouring widths up to 7/8 bits (the appendix sweeps the ratio of
                               two widths)                                                         */
} tahq_config;

/* Fill *cfg with the defaults (tile 64, budget 3.8, tau 2.0, eps 1e-8, scope 0,
 * dtype bf16, dimensions 0).  cfg: host, written.  No error: NULL is ignored. */
void tahq_config_default(tahq_config *cfg);

/* Number of wide (lo+1 bit, 4-bit by default) allocation tiles per ranking unit:
 * round((budget_bits - lo) * n) with n
 * the allocation tiles of one sample (scope 0) or of the tensor (scope 1)  [Sec. 3.2, top-p%].
 * Returns 0 for an invalid cfg (a valid cfg with budget 3.0 also gives 0). */
uint64_t tahq_k_per_unit(const tahq_config *cfg);

/* Size in bytes of the encoded stream; depends on cfg only  [Sec. 3.4: the
 * communication layer sees a fixed-shape buffer].  0 if cfg is invalid. */
size_t tahq_packed_size(const tahq_config *cfg);

/* Bytes of device scratch that tahq_encode needs (tahq_decode uses none).
 * 0 if cfg is invalid. */
size_t tahq_workspace_size(const tahq_config *cfg);

/* Encode  [Sec. 3.1-3.4].
 *   d_in        device, read:    B*S*C elements of cfg->dtype
 *   d_packed    device, written: tahq_packed_size(cfg) bytes (every byte, padding included)
 *   packed_capacity              bytes available at d_packed
 *   d_workspace device, scratch: tahq_workspace_size(cfg) bytes, contents undefined before and after
 * Enqueues on `stream` and returns; the stream is complete when the kernels are. */
tahq_status tahq_encode(const tahq_config *cfg, const void *d_in,
                        void *d_packed, size_t packed_capacity,
                        void *d_workspace, size_t workspace_capacity,
                        tahq_stream stream);

/* tahq_encode for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as
 * tahq_encode, byte for byte; the encoder's scratch is a buffer built into the library (a
 * file-scope device array of TAHQ_NOALLOC_MAX_WORKSPACE bytes that every GPU the library runs on
 * holds until the process ends).  The call allocates nothing and frees nothing.
 *   d_in, d_packed, packed_capacity, stream: as tahq_encode; `stream` must belong to the current device
 * Errors as tahq_encode, and TAHQ_ERR_TOO_LARGE (nothing enqueued) when tahq_workspace_size(cfg)
 * exceeds TAHQ_NOALLOC_MAX_WORKSPACE.  The first call on a device looks up that device's copy of
 * the buffer (hipGetSymbolAddress); make it outside stream capture.
 * All calls on one GPU share that GPU's buffer: two calls whose kernels may overlap there (different
 * streams, or host threads that do not order their streams) race; order them, or use tahq_encode
 * with a workspace per stream.  tahq_decode needs no scratch and has no such variant. */
#define TAHQ_NOALLOC_MAX_WORKSPACE (32u << 20)
tahq_status tahq_encode_noalloc(const tahq_config *cfg, const void *d_in,
                                void *d_packed, size_t packed_capacity,
                                tahq_stream stream);

/* The encoder's phases, in the order they run.  tahq_encode runs all of them. */
enum {
    TAHQ_PHASE_PROLOGUE = 1,   /* header, section padding, cleared selection scratch          */
    TAHQ_PHASE_ENTROPY = 2,    /* Eq. 1-2 for every tile (skipped when every tile gets one width) */
    TAHQ_PHASE_SELECT = 4,     /* top-p% selection: bit map and rank table     [Sec. 3.2]     */
    TAHQ_PHASE_QUANT = 8,      /* Eq. 3-4, quantize, pack                      [Sec. 3.3-3.4] */
    TAHQ_PHASE_ALL = 15,
    /* Not a phase but an option, OR-ed into `phases`: rank every ranking unit with the general
     * multi-launch selection.  By default one workgroup ranks a unit of up to 32768 tiles in a single
     * launch, and larger units that start on 64-tile boundaries are ranked in two launches from a
     * histogram the entropy phase builds.  Same result; meant for tests and timing.  Pass it with
     * every phase of a call sequence, since the prologue and the entropy phase prepare different
     * scratch for each way. */
    TAHQ_SELECT_MULTI_LAUNCH = 16
};

/* tahq_encode split by phase, so that a caller can put its own events between the
 * phases and time each kernel  [Sec. 3.4: the paper profiles the codec's overhead].
 * `phases` is an OR of TAHQ_PHASE_*; a phase needs the results of the earlier ones, left
 * in d_packed / d_workspace by previous calls with the same cfg and buffers.  Calling it
 * once per phase, in order, on one stream equals tahq_encode.  Other arguments and
 * errors as tahq_encode; no phase bit or unknown bits give TAHQ_ERR_INVALID_ARG. */
tahq_status tahq_encode_phases(const tahq_config *cfg, const void *d_in,
                               void *d_packed, size_t packed_capacity,
                               void *d_workspace, size_t workspace_capacity,
                               uint32_t phases, tahq_stream stream);

/* Decode  [Alg. 1 step 5; Sec. 3.3: apply H^T to the de-quantized values].
 *   d_packed    device, read:    a stream produced by tahq_encode with the same cfg
 *   packed_bytes                 bytes valid at d_packed (>= tahq_packed_size(cfg))
 *   d_out       device, written: B*S*C elements of out_dtype (fp32, or bf16 rounded to nearest even)
 *   d_workspace, workspace_capacity: reserved, not used; pass NULL and 0
 * The stream's header is not read back: cfg is trusted.  The stream's contents are not: a
 * stream damaged in transit decodes to meaningless values, but every address the decoder forms
 * stays inside the stream and the output (the rank table is clamped, the pivot index masked). */
tahq_status tahq_decode(const tahq_config *cfg, const void *d_packed, size_t packed_bytes,
                        void *d_out, uint32_t out_dtype,
                        void *d_workspace, size_t workspace_capacity,
                        tahq_stream stream);

/* Sample-wise use in a pipeline  [Alg. 1 steps 4-5: the sender ships Q(a) to the next stage, which
 * de-quantizes on arrival; Sec. 3.4: the communication layer sees fixed-shape buffers].  With scope 0 every
 * sample is ranked on its own, so a run of samples is a micro-batch of its own: tahq_encode_samples
 * encodes samples [first, first + count) of the tensor at d_in into a SELF-CONTAINED stream -- byte for
 * byte what tahq_encode writes for a tensor [count, seq, hidden] that holds just those samples, header
 * included -- so that it can be sent while later samples are still being encoded (e.g. on another
 * stream, with a workspace of its own), and tahq_decode_samples decodes such a stream into the same
 * samples of the tensor at d_out as soon as it has arrived, whatever happens to the others.
 *   cfg          the whole tensor's configuration (cfg->batch samples); scope must be 0
 *   first, count the samples; first + count <= cfg->batch, count >= 1
 *   d_in / d_out device: base of the WHOLE tensor [batch, seq, hidden]
 *   d_packed     device: the run's stream, tahq_samples_packed_size(cfg, count) bytes
 *   d_workspace  device scratch of tahq_samples_workspace_size(cfg, count) bytes; runs that may be in flight
 *                at the same time need a workspace each
 * Errors as tahq_encode / tahq_decode; TAHQ_ERR_INVALID_ARG for scope 1 or samples outside the tensor. */
size_t tahq_samples_packed_size(const tahq_config *cfg, uint32_t count);
size_t tahq_samples_workspace_size(const tahq_config *cfg, uint32_t count);
tahq_status tahq_encode_samples(const tahq_config *cfg, uint32_t first, uint32_t count, const void *d_in,
                                void *d_packed, size_t packed_capacity,
                                void *d_workspace, size_t workspace_capacity, tahq_stream stream);
tahq_status tahq_decode_samples(const tahq_config *cfg, uint32_t first, uint32_t count,
                                const void *d_packed, size_t packed_bytes,
                                void *d_out, uint32_t out_dtype, tahq_stream stream);

/* Intermediates of the encoder, for tests and profiling  [Sec. 3.2 Eq. 1-2].
 *   d_entropy   device, written: float[T], the entropy of every raw quantization tile
 *               (cfg->alloc_tile is ignored: the result is that of A = G)
 * Same validation as tahq_encode. */
tahq_status tahq_tile_entropy(const tahq_config *cfg, const void *d_in, float *d_entropy,
                              tahq_stream stream);

/* Entropy of every allocation tile of A = cfg->alloc_tile channels  [Sec. 3.2 Eq. 1-2 on
 * the reshaped tensor B x (S*C/A) x A]: the values the encoder ranks.
 *   d_entropy   device, written: float[B*S*C/A]
 *   d_workspace device, scratch: tahq_workspace_size(cfg) bytes (used only when A > G)
 * Same validation as tahq_encode. */
tahq_status tahq_alloc_tile_entropy(const tahq_config *cfg, const void *d_in, float *d_entropy,
                                    void *d_workspace, size_t workspace_capacity, tahq_stream stream);

/* Parse the 64-byte header of a stream that was copied to the host.
 *   header64    host, read: the first 64 bytes of a stream
 *   cfg         host, written: the configuration the stream was encoded with
 * Returns TAHQ_ERR_INVALID_ARG if the magic or version does not match. */
tahq_status tahq_parse_header(const void *header64, tahq_config *cfg);

/* Static, NUL-terminated description of a status code. */
const char *tahq_status_string(tahq_status s);

/* Library version: (major << 16) | minor. */
uint32_t tahq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TAHQ_H */
