/*
 * Oracle of the backward-pass compressor Q_Naive with gradient pre-scaling -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow C99 written from the paper: Sec. 3.5 / Alg. 1 steps 6-7 (the backward pass sends
 * activation gradients through a "simple fixed-point" b-bit compressor, 6-8 bits in the main text,
 * 4 and 10 bits in the appendix on backward quantization) and the appendix's gradient-scaling
 * equation g_hat = Q(c g) / c with a constant factor c.  Nothing here is shared with the HIP
 * library; only tests, the smoke check and the benchmark's CPU baseline may call it.
 *
 * The paper gives no formula for Q_Naive.  Reading taken (fixed point in the literal sense):
 *   q     = clamp(round_half_even(c * g), -2^(b-1), 2^(b-1) - 1)      a b-bit two's-complement integer
 *   g_hat = q * (1/c)
 * i.e. the step of the grid is the constant 1/c, there is no data-dependent scale and no metadata, which
 * is why c matters for gradients of magnitude 1e-5.  All arithmetic is IEEE binary32: y = c*g is one
 * rounded multiply; 1/c is rounded once (so "/ c" is exact whenever c is a power of two); a NaN
 * product takes the lower clamp bound (fmaxf/fminf return their non-NaN operand).
 *
 * Stream: 64-byte header ("TAHN", version 1, dtype, B, S, C, b, bits of c; little-endian 32-bit words,
 * rest zero), then the codes of all B*S*C elements in storage order as one LSB-first bit string:
 * element i occupies bits [b*i, b*i + b) of the payload, as q mod 2^b.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

typedef struct {
    uint32_t batch, seq, hidden;   /* B, S, C: contiguous row-major tensor                    */
    uint32_t dtype;                /* 0 = fp32, 1 = bf16 (bit patterns in uint16)             */
    uint32_t bits;                 /* b in [2, 16]                                             */
    float scale;                   /* c of g_hat = Q(c g)/c: finite, > 0                       */
} naive_oracle_cfg;

static int cfg_ok(const naive_oracle_cfg *c)
{
    if (!c || c->batch == 0 || c->seq == 0 || c->hidden == 0) return 0;
    if (c->hidden % 32) return 0;          /* 32 codes always fill whole 32-bit words */
    if (c->dtype > 1) return 0;
    if (c->bits < 2 || c->bits > 16) return 0;
    if (!(c->scale > 0.0f) || isinf(c->scale)) return 0;
    return 1;
}

static uint64_t n_elements(const naive_oracle_cfg *c) { return (uint64_t)c->batch * c->seq * c->hidden; }

uint64_t naive_oracle_packed_size(const naive_oracle_cfg *c)
{
    if (!cfg_ok(c)) return 0;
    return 64 + n_elements(c) * c->bits / 8;
}

static float load_element(const naive_oracle_cfg *c, const void *in, uint64_t i)
{
    if (c->dtype == 0) return ((const float *)in)[i];
    uint32_t u = (uint32_t)((const uint16_t *)in)[i] << 16;     /* bf16 widens exactly */
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32 -> bf16, round to nearest even; NaN stays NaN. */
static uint16_t bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* The quantizer itself: one element. */
int32_t naive_oracle_code(float g, float scale, uint32_t bits)
{
    float lo = -(float)(1u << (bits - 1));
    float hi = (float)((1u << (bits - 1)) - 1u);
    float y = scale * g;
    float r = rintf(y);              /* round half to even (default rounding mode) */
    r = fmaxf(r, lo);
    r = fminf(r, hi);
    return (int32_t)r;
}

float naive_oracle_value(int32_t q, float scale)
{
    float rc = 1.0f / scale;
    return (float)q * rc;
}

int naive_oracle_encode(const naive_oracle_cfg *c, const void *in, uint8_t *packed, uint64_t capacity)
{
    if (!cfg_ok(c) || !in || !packed) return 1;
    uint64_t total = naive_oracle_packed_size(c);
    if (capacity < total) return 2;
    memset(packed, 0, (size_t)total);
    uint32_t hdr[16];
    memset(hdr, 0, sizeof hdr);
    hdr[0] = 0x4e484154u;            /* "TAHN" */
    hdr[1] = 1;
    hdr[2] = c->dtype; hdr[3] = c->batch; hdr[4] = c->seq; hdr[5] = c->hidden; hdr[6] = c->bits;
    memcpy(&hdr[7], &c->scale, 4);
    for (int w = 0; w < 16; ++w)
        for (int k = 0; k < 4; ++k) packed[4 * w + k] = (uint8_t)(hdr[w] >> (8 * k));
    uint8_t *pay = packed + 64;
    uint64_t N = n_elements(c);
    uint32_t b = c->bits;
    for (uint64_t i = 0; i < N; ++i) {
        int32_t q = naive_oracle_code(load_element(c, in, i), c->scale, b);
        uint32_t field = (uint32_t)q & ((1u << b) - 1u);
        uint64_t bit = (uint64_t)b * i;
        for (uint32_t t = 0; t < b; ++t)
            if ((field >> t) & 1u) pay[(bit + t) >> 3] |= (uint8_t)(1u << ((bit + t) & 7));
    }
    return 0;
}

int naive_oracle_decode(const naive_oracle_cfg *c, const uint8_t *packed, uint64_t bytes, void *out,
                        uint32_t out_dtype)
{
    if (!cfg_ok(c) || !packed || !out || out_dtype > 1) return 1;
    if (bytes < naive_oracle_packed_size(c)) return 2;
    const uint8_t *pay = packed + 64;
    uint64_t N = n_elements(c);
    uint32_t b = c->bits;
    for (uint64_t i = 0; i < N; ++i) {
        uint64_t bit = (uint64_t)b * i;
        uint32_t field = 0;
        for (uint32_t t = 0; t < b; ++t)
            field |= (uint32_t)((pay[(bit + t) >> 3] >> ((bit + t) & 7)) & 1u) << t;
        int32_t q = (int32_t)field;
        if (field & (1u << (b - 1))) q -= (int32_t)(1u << b);          /* two's complement */
        float v = naive_oracle_value(q, c->scale);
        if (out_dtype == 0) ((float *)out)[i] = v;
        else ((uint16_t *)out)[i] = bf16_rne(v);
    }
    return 0;
}
