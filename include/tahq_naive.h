/*
 * tahq_naive -- the backward-pass compressor of TAH-Quant's pipeline for AMD MI355X (gfx950).
 *
 * Part of libtahq.so.  In the paper's pipeline-parallel loop the activation gradients travel
 * back through a "simple fixed-point" b-bit compressor Q_Naive (6-8 bits in the main text, 4 and
 * 10 bits in the appendix on backward quantization)            [Sec. 3.5, Alg. 1 steps 6-7],
 * applied to gradients that are rescaled by a constant c first:
 * g_hat = Q(c g) / c                                           [appendix, gradient scaling].
 *
 * The paper gives no formula for Q_Naive; this library takes fixed point literally:
 *     q     = clamp(round_half_even(c * g), -2^(b-1), 2^(b-1) - 1)
 *     g_hat = q * (1/c)
 * in IEEE binary32 (c*g is one rounded multiply, 1/c is rounded once, so "/ c" is exact when c
 * is a power of two; a NaN product takes the lower bound).  There is no data-dependent scale
 * and no metadata: the step of the grid is the constant 1/c.
 *
 * Stream (little-endian): 64-byte header ("TAHN", version 1, dtype, batch, seq, hidden, b, the
 * bits of c; 32-bit words, rest zero), then the codes of all elements in storage order as one
 * LSB-first bit string: element i occupies bits [b*i, b*i + b) as q mod 2^b.
 *
 * Conventions as in tahq.h: d_* are DEVICE pointers, 16-byte aligned, owned by the caller and
 * not overlapping; cfg is a HOST pointer; the library allocates nothing, never synchronizes,
 * validates on the host and then only enqueues kernels on `stream`; status codes are tahq_status.
 */
#ifndef TAHQ_NAIVE_H
#define TAHQ_NAIVE_H

#include "tahq.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    uint32_t struct_size;   /* = sizeof(tahq_naive_config); set by tahq_naive_config_default     */
    uint32_t batch;         /* B                                                                  */
    uint32_t seq;           /* S                                                                  */
    uint32_t hidden;        /* C, a multiple of 32; tensor is contiguous row-major [B, S, C]      */
    uint32_t dtype;         /* tahq_dtype of the gradient tensor                                  */
    uint32_t bits;          /* b, the code width: 2 .. 16                                         */
    float scale;            /* c of g_hat = Q(c g)/c: finite and > 0; default 1.0                 */
} tahq_naive_config;

/* Defaults: 8 bits, c = 1, bf16, dimensions 0.  cfg: host, written; NULL is ignored. */
void tahq_naive_config_default(tahq_naive_config *cfg);

/* 64 + B*S*C*b/8: depends on cfg only  [Sec. 3.4: a fixed-shape buffer].  0 if cfg is invalid
 * (zero dimension, hidden % 32 != 0, b outside 2..16, c not finite or not positive, bad dtype,
 * more than 2^36 elements). */
size_t tahq_naive_packed_size(const tahq_naive_config *cfg);

/* Q(c g)  [Alg. 1 step 6; appendix, gradient scaling].
 *   d_in      device, read:    B*S*C elements of cfg->dtype
 *   d_packed  device, written: tahq_naive_packed_size(cfg) bytes
 * Errors: TAHQ_ERR_NULL, _INVALID_ARG (bad cfg), _BUFFER_TOO_SMALL, _MISALIGNED, _HIP. */
tahq_status tahq_naive_encode(const tahq_naive_config *cfg, const void *d_in,
                              void *d_packed, size_t packed_capacity, tahq_stream stream);

/* q / c  [Alg. 1 step 7; appendix, gradient scaling].
 *   d_packed  device, read:    a stream produced by tahq_naive_encode with the same cfg
 *   d_out     device, written: B*S*C elements of out_dtype (fp32, or bf16 rounded to nearest even)
 * The stream's header is not read back: cfg is trusted.  Errors as tahq_naive_encode;
 * out_dtype outside tahq_dtype gives TAHQ_ERR_INVALID_ARG. */
tahq_status tahq_naive_decode(const tahq_naive_config *cfg, const void *d_packed, size_t packed_bytes,
                              void *d_out, uint32_t out_dtype, tahq_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* TAHQ_NAIVE_H */
