/*
 * TAH-Quant stage-boundary activation codec: CPU oracle (fp32 operation order).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, plain-C
 * statement of what the codec computes.  It shares no code, header, table or
 * constant generator with the HIP library; only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may load it.
 *
 * It follows the paper's Section 3 step by step, in the paper's notation:
 *   Sec. 3.1   tile-wise group quantization (tiles of G contiguous channels)
 *   Sec. 3.2   Eq. 1 (p_k), Eq. 2 (entropy H), top-p% tile selection
 *   Sec. 3.3   Eq. 3 (outlier ratio r vs tau), pivot swap P_d, Eq. 4
 *              (Hadamard transform), asymmetric uniform quantization
 *   Sec. 3.4   packing into one contiguous uint8 stream of fixed shape
 *   Alg. 1     step 5: dequantize (inverse of every step)
 *
 * Where the paper leaves a choice open the reading taken is stated at the
 * function that needs it.  All floating point is IEEE binary32 with no
 * contraction; fmaf() appears only where the numerics contract writes a fused
 * multiply-add.  Build: gcc -O2 -std=c99 -ffp-contract=off (no -ffast-math).
 *
 * Pins (tests, "not gpu"): every function below is checked against something
 * other than itself -- dense Sylvester matrices, closed-form entropies,
 * brute-force subset search, numpy float16, a textbook min-max group
 * quantizer, an independent float64 decoder of the byte stream.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- config */

typedef struct {
    uint32_t batch;       /* B */
    uint32_t seq;         /* S */
    uint32_t hidden;      /* C */
    uint32_t tile;        /* G = A (Sec. 3.2: default A = G) */
    uint32_t dtype;       /* 0 = fp32, 1 = bf16 (of the activation tensor) */
    uint32_t scope;       /* 0 = rank the tiles of every sample (Sec. 3.2); 1 = rank the whole tensor */
    float budget_bits;    /* mean payload bits per element, in [lo, lo+1]; p% = budget-lo (lo = 3 by default) */
    float tau;            /* Eq. 3 threshold */
    float eps_l1;         /* epsilon of Eq. 1 */
    float eps_log;        /* varsigma of Eq. 2 */
    float eps_ratio;      /* varrho of Eq. 3 */
    uint32_t alloc_tile;  /* A: allocation-tile size (Sec. 3.2), a multiple of G dividing C; 0 means A = G */
    uint32_t low_bits;    /* lo: the two widths are lo and lo+1, 1 <= lo <= 7.  3 (or 0) = INT3/INT4, the paper's
                             setting; 2 = the INT2/INT3 mix of the appendix on bit allocation; the same appendix
                             sweeps the ratio of two neighbouring widths, which any lo gives */
} tahq_oracle_cfg;

enum { OR_OK = 0, OR_BAD = 1, OR_SMALL = 2 };

static int cfg_ok(const tahq_oracle_cfg *c)
{
    if (!c) return 0;
    if (c->batch == 0 || c->seq == 0 || c->hidden == 0) return 0;
    if (c->tile != 8 && c->tile != 16 && c->tile != 32 && c->tile != 64 && c->tile != 128) return 0;
    if (c->hidden % c->tile) return 0;
    if (c->dtype > 1 || c->scope > 1) return 0;
    if (c->low_bits > 7) return 0;
    float lo = c->low_bits ? (float)c->low_bits : 3.0f;
    if (!(c->budget_bits >= lo && c->budget_bits <= lo + 1.0f)) return 0;
    if (c->alloc_tile != 0 && (c->alloc_tile % c->tile || c->hidden % c->alloc_tile)) return 0;
    return 1;
}

/* lo: the narrower of the two code widths. */
static uint32_t low_bits(const tahq_oracle_cfg *c) { return c->low_bits ? c->low_bits : 3u; }

/* m = A / G: quantization tiles per allocation tile (Sec. 3.2: A is aligned with the quantization tiles). */
static uint32_t tiles_per_alloc(const tahq_oracle_cfg *c)
{
    return c->alloc_tile ? c->alloc_tile / c->tile : 1u;
}

static uint64_t n_tiles(const tahq_oracle_cfg *c)
{
    return (uint64_t)c->batch * c->seq * (c->hidden / c->tile);
}

/* Ranking unit: one sample (scope 0) or the whole tensor (scope 1).  Counted in quantization tiles. */
static uint64_t tiles_per_unit(const tahq_oracle_cfg *c)
{
    uint64_t n = (uint64_t)c->seq * (c->hidden / c->tile);
    return c->scope ? n * c->batch : n;
}
/* ... and in allocation tiles: the S*M tiles of Sec. 3.2 that are ranked. */
static uint64_t alloc_tiles_per_unit(const tahq_oracle_cfg *c)
{
    return tiles_per_unit(c) / tiles_per_alloc(c);
}
static uint64_t n_units(const tahq_oracle_cfg *c) { return c->scope ? 1 : c->batch; }

/* Sec. 3.2, top-p%: number of wide (lo+1 bit, INT4 by default) allocation tiles per ranking unit.  p = budget-lo,
 * so the mean payload width is 3 + k/n.  Rounded to nearest, in double. */
uint64_t tahq_oracle_k(const tahq_oracle_cfg *c)
{
    double n = (double)alloc_tiles_per_unit(c);
    double k = floor((double)c->budget_bits * n - (double)low_bits(c) * n + 0.5);
    if (k < 0) k = 0;
    if (k > n) k = n;
    return (uint64_t)k;
}

/* ------------------------------------------------------- small numerics */

static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* bf16 is the upper half of an fp32: widening is exact. */
static float bf16_widen(uint16_t h) { return bits_f32((uint32_t)h << 16); }

/* fp32 -> bf16, round to nearest even (finite inputs). */
uint16_t tahq_oracle_bf16_rne(float f)
{
    uint32_t u = f32_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN stays NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* IEEE binary16 <-> binary32, written out bit by bit. */
float tahq_oracle_fp16_widen(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t ex = (h >> 10) & 0x1fu;
    uint32_t man = h & 0x3ffu;
    if (ex == 0) {
        /* zero or subnormal: man * 2^-24, exact in fp32 */
        float v = (float)man * 0x1p-24f;
        return (sign ? -v : v);
    }
    if (ex == 31) return bits_f32(sign | 0x7f800000u | (man << 13));
    return bits_f32(sign | ((ex + 112u) << 23) | (man << 13));
}

/* fp32 -> binary16, round to nearest even, subnormals kept. */
uint16_t tahq_oracle_fp16_rne(float f)
{
    uint32_t u = f32_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);       /* NaN */
    if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);      /* >= 65520 rounds to inf */
    if (a < 0x33000001u) return sign;                             /* <= 2^-25 rounds to zero */
    int e = (int)(a >> 23) - 127;                                 /* unbiased exponent */
    uint32_t m = (a & 0x7fffffu) | 0x800000u;                     /* 24-bit significand */
    int shift;                                                    /* bits dropped from m */
    uint32_t base;
    if (e >= -14) { shift = 13; base = (uint32_t)(e + 15) << 10; m &= 0x7fffffu; }
    else { shift = 13 + (-14 - e); base = 0; }                    /* subnormal result */
    uint32_t q = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (q & 1u))) q += 1;          /* carries ripple into the exponent */
    return (uint16_t)(sign | (base + q));
}

/* One step towards -inf / +inf on the binary16 number line (finite values). */
static uint16_t fp16_prev(uint16_t h)
{
    if (h == 0x0000u || h == 0x8000u) return 0x8001u;
    return (h & 0x8000u) ? (uint16_t)(h + 1) : (uint16_t)(h - 1);
}
static uint16_t fp16_next(uint16_t h)
{
    if (h == 0x0000u || h == 0x8000u) return 0x0001u;
    return (h & 0x8000u) ? (uint16_t)(h - 1) : (uint16_t)(h + 1);
}

static float clamp_fp16_range(float x)
{
    /* fmaxf/fminf drop a NaN operand; metadata saturates at +-65504. */
    return fminf(fmaxf(x, -65504.0f), 65504.0f);
}

/* Largest binary16 <= x (after saturating x to +-65504): the stored zero-point. */
uint16_t tahq_oracle_fp16_down(float x)
{
    float xc = clamp_fp16_range(x);
    uint16_t h = tahq_oracle_fp16_rne(xc);
    if (tahq_oracle_fp16_widen(h) > xc) h = fp16_prev(h);
    if (h == 0x8000u) h = 0x0000u;
    return h;
}

/* Smallest binary16 >= x (after saturating): the stored scale. */
uint16_t tahq_oracle_fp16_up(float x)
{
    float xc = clamp_fp16_range(x);
    uint16_t h = tahq_oracle_fp16_rne(xc);
    if (tahq_oracle_fp16_widen(h) < xc) h = fp16_next(h);
    if (h == 0x8000u) h = 0x0000u;
    return h;
}

/* Natural logarithm as the numerics contract fixes it (Eq. 2 needs log(p+varsigma)):
 * u = m * 2^e with m in [0.5,1); ln u = e*ln2 + P(m), P a degree-5 polynomial
 * evaluated by Horner's rule with fused multiply-adds.  |LOG(u) - ln u| <= 1.1e-5. */
float tahq_oracle_log(float u)
{
    int e;
    float m = frexpf(u, &e);
    float P = 0x1.00ef0ap+0f;
    P = fmaf(P, m, -0x1.29aa42p+2f);
    P = fmaf(P, m, 0x1.22ea48p+3f);
    P = fmaf(P, m, -0x1.3c1c5cp+3f);
    P = fmaf(P, m, 0x1.c4859ep+2f);
    P = fmaf(P, m, -0x1.5165a2p+1f);
    return fmaf((float)e, 0x1.62e430p-1f, P);
}

/* Sum by the adjacent-pair binary tree: level by level z'[k] = z[2k] + z[2k+1].
 * n is a power of two; z is overwritten. */
static float tree_sum(float *z, uint32_t n)
{
    while (n > 1) {
        n >>= 1;
        for (uint32_t k = 0; k < n; ++k) z[k] = z[2 * k] + z[2 * k + 1];
    }
    return z[0];
}

/* Eq. 1 and Eq. 2 on one allocation tile of m quantization tiles (A = m*G channels, Sec. 3.2; m = 1 in
 * the default configuration A = G).  Eq. 2 is printed without a minus sign, yet the text beside it says H
 * is high for evenly spread energy and low for a sharp outlier; that fixes H = -sum p log(p+varsigma)
 * (Shannon), natural log.  The norm and the entropy are sums over the A channels: inside each
 * quantization tile by the pairwise tree, and across the m tiles from left to right.
 * Order of evaluation: with r = 1/(L1 + eps) the probability is p = |v| r, and the common factor r is taken out
 * of Eq. 2's sum: H = -r * sum |v| log(|v| r + varsigma), the argument of the logarithm being one fused
 * multiply-add. */
float tahq_oracle_entropy_alloc(const float *v, uint32_t G, uint32_t m, float eps_l1, float eps_log)
{
    float w[128];
    float L1 = 0.0f;
    for (uint32_t q = 0; q < m; ++q) {
        for (uint32_t k = 0; k < G; ++k) w[k] = fabsf(v[q * G + k]);
        L1 = L1 + tree_sum(w, G);
    }
    float invL = 1.0f / (L1 + eps_l1);
    float W = 0.0f;
    for (uint32_t q = 0; q < m; ++q) {
        for (uint32_t k = 0; k < G; ++k) {
            float a = fabsf(v[q * G + k]);
            float u = fmaf(a, invL, eps_log);
            w[k] = a * tahq_oracle_log(u);
        }
        W = W + tree_sum(w, G);
    }
    return 0.0f - invL * W;
}

/* The default A = G: the allocation tile is the quantization tile. */
float tahq_oracle_entropy(const float *v, uint32_t G, float eps_l1, float eps_log)
{
    return tahq_oracle_entropy_alloc(v, G, 1, eps_l1, eps_log);
}

/* Eq. 3: pivot index d (lowest index among equal maxima), and whether the
 * ratio exceeds tau.  "Exceeds" is read as strict; the test is written without
 * the division, |a(1)| > tau * (|a(2)| + varrho).  The second-largest counts
 * multiplicity: two equal maxima give r ~ 1. */
int tahq_oracle_outlier(const float *v, uint32_t G, float tau, float eps_ratio, uint32_t *d_out)
{
    uint32_t d = 0;
    float a1 = fabsf(v[0]);
    for (uint32_t k = 1; k < G; ++k)
        if (fabsf(v[k]) > a1) { a1 = fabsf(v[k]); d = k; }
    float a2 = 0.0f;
    for (uint32_t k = 0; k < G; ++k)
        if (k != d && fabsf(v[k]) > a2) a2 = fabsf(v[k]);
    float t = a2 + eps_ratio;
    float t2 = tau * t;
    *d_out = d;
    return a1 > t2;
}

/* Unnormalised Sylvester-Hadamard butterfly, natural order: stages h = 1, 2,
 * ..., G/2; in each, (x, y) -> (x + y, x - y) for the pairs h apart. */
void tahq_oracle_butterfly(float *v, uint32_t G)
{
    for (uint32_t h = 1; h < G; h <<= 1)
        for (uint32_t i = 0; i < G; i += 2 * h)
            for (uint32_t j = i; j < i + h; ++j) {
                float x = v[j], y = v[j + h];
                v[j] = x + y;
                v[j + h] = x - y;
            }
}

/* fp32(1/sqrt(G)) for the supported tile widths. */
static float c_G(uint32_t G)
{
    switch (G) {
    case 8: return 0x1.6a09e6p-2f;
    case 16: return 0.25f;
    case 32: return 0x1.6a09e6p-3f;
    case 64: return 0.125f;
    default: return 0x1.6a09e6p-4f;      /* 128 */
    }
}

/* Sec. 3.3, Eq. 4: alpha P_d (1/sqrt(G)) H_G.  P_d swaps coordinates 1 and d. */
void tahq_oracle_forward_transform(float *v, uint32_t G, uint32_t d)
{
    float t = v[0]; v[0] = v[d]; v[d] = t;
    tahq_oracle_butterfly(v, G);
    float c = c_G(G);
    for (uint32_t k = 0; k < G; ++k) v[k] = v[k] * c;
}

/* Inverse: H is symmetric and P_d is an involution, so the same butterfly,
 * the same scale, then the same swap. */
void tahq_oracle_inverse_transform(float *v, uint32_t G, uint32_t d)
{
    tahq_oracle_butterfly(v, G);
    float c = c_G(G);
    for (uint32_t k = 0; k < G; ++k) v[k] = v[k] * c;
    float t = v[0]; v[0] = v[d]; v[d] = t;
}

/* Per-tile record of everything the encoder derives before widths are known. */
typedef struct {
    float H;          /* Eq. 2 on the raw tile */
    float mn, mx;     /* range of the tile that will be quantized (+0 canonical) */
    uint8_t pivot;    /* bit 7 = transformed, bits 0..6 = d (0 if not transformed) */
} tile_rec;

static void load_tile(const tahq_oracle_cfg *c, const void *in, uint64_t j, float *v)
{
    uint32_t G = c->tile;
    if (c->dtype == 0) {
        const float *p = (const float *)in + j * G;
        for (uint32_t k = 0; k < G; ++k) v[k] = p[k];
    } else {
        const uint16_t *p = (const uint16_t *)in + j * G;
        for (uint32_t k = 0; k < G; ++k) v[k] = bf16_widen(p[k]);
    }
}

/* Steps 1-4 for tile j: entropy of the raw tile, outlier test, conditional
 * swap + Hadamard, range.  On return y[] holds the tile in the domain that is
 * quantized (transformed or raw, Sec. 3.3 "asymmetric uniform quantization"). */
static void analyse_tile(const tahq_oracle_cfg *c, const float *v, float *y, tile_rec *r)
{
    uint32_t G = c->tile, d = 0;
    r->H = tahq_oracle_entropy(v, G, c->eps_l1, c->eps_log);
    int flag = tahq_oracle_outlier(v, G, c->tau, c->eps_ratio, &d);
    for (uint32_t k = 0; k < G; ++k) y[k] = v[k];
    if (flag) tahq_oracle_forward_transform(y, G, d);
    float mn = y[0], mx = y[0];
    for (uint32_t k = 1; k < G; ++k) { mn = fminf(mn, y[k]); mx = fmaxf(mx, y[k]); }
    r->mn = mn + 0.0f;   /* -0 -> +0, so metadata bytes cannot depend on which zero min/max returned */
    r->mx = mx + 0.0f;
    r->pivot = flag ? (uint8_t)(0x80u | d) : 0;
}

/* The asymmetric uniform quantizer (the paper only cites it): min/max affine
 * with 2^b - 1 steps, real-valued zero-point = tile minimum, round half to even,
 * clamp.  Scale and zero-point travel as binary16, rounded outwards (zero-point
 * down, scale up), so that the coded range [z, z + L s] covers [mn, mx] up to the
 * one binary32 rounding of (mx - z) / L: the top of the range may fall short of
 * mx by a fraction 2^-22 of (mx - z), and the clamp takes care of that. */
void tahq_oracle_quant_params(float mn, float mx, uint32_t b, uint16_t *s16, uint16_t *z16)
{
    float Lv = (float)((1u << b) - 1u);
    uint16_t z = tahq_oracle_fp16_down(mn);
    float mnf = tahq_oracle_fp16_widen(z);
    float s = (mx - mnf) / Lv;
    uint16_t sh = tahq_oracle_fp16_up(s);
    if ((sh & 0x7fffu) == 0) sh = 0x3c00u;   /* constant tile: scale 1, every code 0 */
    *s16 = sh;
    *z16 = z;
}

uint32_t tahq_oracle_quant_code(float y, uint16_t s16, uint16_t z16, uint32_t b)
{
    float Lv = (float)((1u << b) - 1u);
    float sf = tahq_oracle_fp16_widen(s16);
    float mnf = tahq_oracle_fp16_widen(z16);
    float r = 1.0f / sf;
    float t = (y - mnf) * r;
    float q = fminf(fmaxf(rintf(t), 0.0f), Lv);   /* rintf: round half to even; a NaN becomes 0 */
    return (uint32_t)q;
}

float tahq_oracle_dequant(uint32_t q, uint16_t s16, uint16_t z16)
{
    return fmaf((float)q, tahq_oracle_fp16_widen(s16), tahq_oracle_fp16_widen(z16));
}

/* ------------------------------------------------------------ byte format */
/* Little-endian; every section padded to 64 bytes, in this order:
 *   header   64 B
 *   bitmap   T bits: tile j -> byte j>>3, bit j&7; 1 = INT4
 *   ranks    uint32[ceil(T/64)]: wide (lo+1 bit) tiles before each group of 64 tiles
 *   pivot    uint8[T]
 *   scale    binary16[T]
 *   zero     binary16[T]
 *   payload  tile j at byte (G/8)*(lo*j + rank(j)), G*b/8 bytes, element k in
 *            bits [b*k, b*k+b) of the tile's LSB-first bit string
 * The shape depends on the configuration only (Sec. 3.4: a fixed-shape buffer). */

static uint64_t pad64(uint64_t x) { return (x + 63u) & ~(uint64_t)63u; }

typedef struct { uint64_t bitmap, ranks, pivot, scale, zero, payload, total; } layout;

static void make_layout(const tahq_oracle_cfg *c, layout *L)
{
    uint64_t T = n_tiles(c);
    uint64_t k = tahq_oracle_k(c);
    L->bitmap = 64;
    L->ranks = L->bitmap + pad64((T + 7) / 8);
    L->pivot = L->ranks + pad64(4 * ((T + 63) / 64));
    L->scale = L->pivot + pad64(T);
    L->zero = L->scale + pad64(2 * T);
    L->payload = L->zero + pad64(2 * T);
    L->total = L->payload + (uint64_t)(c->tile / 8) * (low_bits(c) * T + n_units(c) * k * tiles_per_alloc(c));
}

uint64_t tahq_oracle_packed_size(const tahq_oracle_cfg *c)
{
    if (!cfg_ok(c)) return 0;
    layout L; make_layout(c, &L);
    return L.total;
}

static void put_u32(uint8_t *p, uint32_t v)
{
    p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24);
}
static void put_u16(uint8_t *p, uint16_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static uint32_t get_u32(const uint8_t *p)
{
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}
static uint16_t get_u16(const uint8_t *p) { return (uint16_t)(p[0] | (p[1] << 8)); }

static void write_header(const tahq_oracle_cfg *c, uint8_t *p)
{
    memset(p, 0, 64);
    p[0] = 'T'; p[1] = 'A'; p[2] = 'H'; p[3] = 'Q';
    put_u32(p + 4, 1);
    put_u32(p + 8, c->dtype);
    put_u32(p + 12, c->batch);
    put_u32(p + 16, c->seq);
    put_u32(p + 20, c->hidden);
    put_u32(p + 24, c->tile);
    put_u32(p + 28, c->scope);
    put_u32(p + 32, (uint32_t)tahq_oracle_k(c));
    put_u32(p + 36, f32_bits(c->budget_bits));
    put_u32(p + 40, f32_bits(c->tau));
    put_u32(p + 44, f32_bits(c->eps_l1));
    put_u32(p + 48, f32_bits(c->eps_log));
    put_u32(p + 52, f32_bits(c->eps_ratio));
    put_u32(p + 56, c->alloc_tile ? c->alloc_tile : c->tile);
    put_u32(p + 60, low_bits(c));
}

/* --------------------------------------------------------- bit allocation */

typedef struct { float H; uint64_t j; } rank_item;

static int by_entropy_desc_then_index(const void *pa, const void *pb)
{
    const rank_item *a = (const rank_item *)pa, *b = (const rank_item *)pb;
    if (a->H > b->H) return -1;
    if (a->H < b->H) return 1;
    return (a->j > b->j) - (a->j < b->j);
}

/* Sec. 3.2, top-p% tile selection: inside each ranking unit the k allocation tiles of highest entropy
 * get 4 bits, the rest 3; equal entropies go to the lower tile index.  H has one entry per allocation
 * tile; width[j] receives 3 or 4 for every QUANTIZATION tile j (the m tiles of an allocation tile share
 * its width). */
int tahq_oracle_allocate(const tahq_oracle_cfg *c, const float *H, uint8_t *width)
{
    if (!cfg_ok(c)) return OR_BAD;
    uint64_t n = alloc_tiles_per_unit(c), U = n_units(c), k = tahq_oracle_k(c);
    uint32_t m = tiles_per_alloc(c), lo = low_bits(c);
    rank_item *it = (rank_item *)malloc((size_t)n * sizeof *it);
    if (!it) return OR_BAD;
    for (uint64_t u = 0; u < U; ++u) {
        for (uint64_t j = 0; j < n; ++j) { it[j].H = H[u * n + j]; it[j].j = j; }
        qsort(it, (size_t)n, sizeof *it, by_entropy_desc_then_index);
        for (uint64_t r = 0; r < n; ++r)
            for (uint32_t q = 0; q < m; ++q) width[(u * n + it[r].j) * m + q] = (uint8_t)((r < k) ? lo + 1 : lo);
    }
    free(it);
    return OR_OK;
}

/* Entropy of every allocation tile (T/m values). */
int tahq_oracle_alloc_entropies(const tahq_oracle_cfg *c, const void *in, float *H)
{
    if (!cfg_ok(c) || !in || !H) return OR_BAD;
    uint64_t T = n_tiles(c);
    uint32_t G = c->tile, m = tiles_per_alloc(c);
    float *v = (float *)malloc((size_t)m * G * sizeof(float));
    if (!v) return OR_BAD;
    for (uint64_t ja = 0; ja < T / m; ++ja) {
        for (uint32_t q = 0; q < m; ++q) load_tile(c, in, ja * m + q, v + q * G);
        H[ja] = tahq_oracle_entropy_alloc(v, G, m, c->eps_l1, c->eps_log);
    }
    free(v);
    return OR_OK;
}

/* Steps 1-4 for every tile, exported so tests can look at the intermediates. */
int tahq_oracle_tile_stats(const tahq_oracle_cfg *c, const void *in,
                           float *H, uint8_t *pivot, float *mn, float *mx)
{
    if (!cfg_ok(c) || !in) return OR_BAD;
    uint64_t T = n_tiles(c);
    float v[128], y[128];
    tile_rec r;
    for (uint64_t j = 0; j < T; ++j) {
        load_tile(c, in, j, v);
        analyse_tile(c, v, y, &r);
        if (H) H[j] = r.H;
        if (pivot) pivot[j] = r.pivot;
        if (mn) mn[j] = r.mn;
        if (mx) mx[j] = r.mx;
    }
    return OR_OK;
}

/* ------------------------------------------------------------------ encode */

int tahq_oracle_encode(const tahq_oracle_cfg *c, const void *in, uint8_t *packed, uint64_t cap)
{
    if (!cfg_ok(c) || !in || !packed) return OR_BAD;
    layout L; make_layout(c, &L);
    if (cap < L.total) return OR_SMALL;
    uint64_t T = n_tiles(c);
    uint32_t G = c->tile, lo = low_bits(c);

    float *H = (float *)malloc((size_t)T * sizeof(float));
    uint8_t *width = (uint8_t *)malloc((size_t)T);
    if (!H || !width) { free(H); free(width); return OR_BAD; }

    /* pass 1: entropies of the allocation tiles (Eq. 1-2) */
    float v[128], y[128];
    tile_rec r;
    if (tahq_oracle_alloc_entropies(c, in, H) != OR_OK) { free(H); free(width); return OR_BAD; }
    /* top-p% selection */
    tahq_oracle_allocate(c, H, width);

    memset(packed, 0, (size_t)L.total);
    write_header(c, packed);

    /* pass 2: transform, quantize, pack */
    uint64_t rank = 0;   /* wide (lo+1 bit) tiles before tile j */
    for (uint64_t j = 0; j < T; ++j) {
        if ((j & 63u) == 0) put_u32(packed + L.ranks + 4 * (j >> 6), (uint32_t)rank);
        uint32_t b = width[j];
        if (b == lo + 1) packed[L.bitmap + (j >> 3)] |= (uint8_t)(1u << (j & 7u));

        load_tile(c, in, j, v);
        analyse_tile(c, v, y, &r);
        packed[L.pivot + j] = r.pivot;

        uint16_t s16, z16;
        tahq_oracle_quant_params(r.mn, r.mx, b, &s16, &z16);
        put_u16(packed + L.scale + 2 * j, s16);
        put_u16(packed + L.zero + 2 * j, z16);

        uint8_t *dst = packed + L.payload + (uint64_t)(G / 8) * (lo * j + rank);
        for (uint32_t k = 0; k < G; ++k) {
            uint32_t q = tahq_oracle_quant_code(y[k], s16, z16, b);
            uint32_t bit = b * k;
            /* a code spans at most two bytes */
            dst[bit >> 3] |= (uint8_t)(q << (bit & 7u));
            if ((bit & 7u) + b > 8) dst[(bit >> 3) + 1] |= (uint8_t)(q >> (8 - (bit & 7u)));
        }
        if (b == lo + 1) ++rank;
    }
    free(H); free(width);
    return OR_OK;
}

/* ------------------------------------------------------------------ decode */

/* Alg. 1 step 5: de-quantize, and for transformed tiles apply H^T and undo P_d.
 * out_dtype: 0 = fp32, 1 = bf16 (round to nearest even). */
int tahq_oracle_decode(const tahq_oracle_cfg *c, const uint8_t *packed, uint64_t bytes,
                       void *out, uint32_t out_dtype)
{
    if (!cfg_ok(c) || !packed || !out || out_dtype > 1) return OR_BAD;
    layout L; make_layout(c, &L);
    if (bytes < L.total) return OR_SMALL;
    uint64_t T = n_tiles(c);
    uint32_t G = c->tile, lo = low_bits(c);
    float y[128];
    for (uint64_t j = 0; j < T; ++j) {
        uint32_t b = ((packed[L.bitmap + (j >> 3)] >> (j & 7u)) & 1u) ? lo + 1 : lo;
        /* rank(j): table entry of the group plus set bits below j inside it */
        uint64_t rank = get_u32(packed + L.ranks + 4 * (j >> 6));
        for (uint64_t i = j & ~(uint64_t)63u; i < j; ++i)
            rank += (packed[L.bitmap + (i >> 3)] >> (i & 7u)) & 1u;
        uint16_t s16 = get_u16(packed + L.scale + 2 * j);
        uint16_t z16 = get_u16(packed + L.zero + 2 * j);
        uint8_t pv = packed[L.pivot + j];
        const uint8_t *src = packed + L.payload + (uint64_t)(G / 8) * (lo * j + rank);
        for (uint32_t k = 0; k < G; ++k) {
            uint32_t bit = b * k;
            uint32_t w = src[bit >> 3];
            if ((bit & 7u) + b > 8) w |= (uint32_t)src[(bit >> 3) + 1] << 8;
            uint32_t q = (w >> (bit & 7u)) & ((1u << b) - 1u);
            y[k] = tahq_oracle_dequant(q, s16, z16);
        }
        if (pv & 0x80u) tahq_oracle_inverse_transform(y, G, pv & 0x7fu);
        if (out_dtype == 0) {
            float *o = (float *)out + j * G;
            for (uint32_t k = 0; k < G; ++k) o[k] = y[k];
        } else {
            uint16_t *o = (uint16_t *)out + j * G;
            for (uint32_t k = 0; k < G; ++k) o[k] = tahq_oracle_bf16_rne(y[k]);
        }
    }
    return OR_OK;
}
