// Shapes, stream layout, workspace layout and the device-side numerics shared by all kernels
// of the TAH-Quant codec (Sec. 3.1-3.4 of the paper; see tahq.hip for the overview).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "tahq.h"

namespace tahq {

// ---------------------------------------------------------------- host side

struct Shape {
    uint32_t B, S, C, G, dtype, scope;
    uint32_t low; // the two code widths are low and low + 1 bits, 1..7 (3 by default, 2 for the INT2/INT3 mix)
    uint32_t A;   // allocation tile (Sec. 3.2), a multiple of G
    uint32_t m;   // quantization tiles per allocation tile, A / G
    uint64_t T;   // quantization tiles in the tensor
    uint64_t n;   // quantization tiles per ranking unit
    uint32_t U;   // ranking units
    uint64_t k;   // wide (low + 1 bit) quantization tiles per ranking unit, m * kA
    uint64_t nA;  // allocation tiles per ranking unit: what the selection ranks
    uint64_t kA;  // wide allocation tiles per ranking unit
};

struct Layout {
    uint64_t bitmap, ranks, pivot, scale, zero, payload, total;
};

constexpr uint32_t kSegTiles = 1024;     // tiles one wavefront handles in the selection kernels
constexpr uint32_t kHistBins = 2048;      // bins of radix digits 1 and 2 (11 bits each)
constexpr uint32_t kDigit0Bins = 1024;    // bins of radix digit 0 (key bits 31..22)
constexpr uint32_t kRadixKeysPerBlock = 8192;
constexpr uint32_t kLinBins = 2048;       // bins of the entropy histogram of the single-launch selection of large units
constexpr uint32_t kSubBins = 1024;       // sub-bins of the bin that holds the threshold (k_select_resolve)
constexpr uint32_t kCandCap = 16384;      // tiles of the threshold bin that the selection keeps in a list, per ranking unit

struct Workspace {
    // offsets in bytes from the workspace base
    uint64_t hist0;      // uint32[U][kDigit0Bins]: first-digit histogram      (zeroed per call)
    uint64_t coarse;     // uint32[U][2][64]: super-bin totals of digits 1, 2   (zeroed per call)
    uint64_t state;      // uint32[U][8] selection state
    uint64_t lin_hist;   // uint32[U][kLinBins]: entropies by linear bin                  (zeroed per call)
    uint64_t fused;      // uint32[U][4]: candidates listed, workgroups done              (zeroed per call)
    uint64_t zero_bytes; // bytes from `hist0` that must be zero before the selection starts
    uint64_t partial;    // uint32[U][2][hb][kHistBins]: per-workgroup histograms of digits 1, 2
    uint64_t keys;       // float[T] entropies
    uint64_t cand;       // uint2[U][kCandCap]: (key, tile) of the tiles in the threshold bin
    uint64_t block_above; // uint32[U][ceil(n / 16384)]: tiles above the threshold bin, per block of 16384 tiles
    uint64_t seg;        // uint32[U][nseg][2]: keys equal to / above the threshold, per segment
    uint64_t sel;        // uint8[T] (only when n % 64 != 0, or A > G)
    uint64_t part;       // float[T]: per-quantization-tile partial sums            (only when A > G)
    uint64_t inv_norm;   // float[T/m]: 1 / (L1 norm + eps) of every allocation tile (only when A > G)
    uint64_t ranks_a;    // uint32[ceil(U*nA/64)]: rank table over allocation tiles  (only when A > G)
    uint64_t total;
    uint32_t nseg;       // segments per ranking unit
    uint32_t hb;         // workgroups per ranking unit in the radix passes
};

inline uint64_t pad64(uint64_t x) { return (x + 63u) & ~uint64_t(63); }
inline uint64_t pad256(uint64_t x) { return (x + 255u) & ~uint64_t(255); }

tahq_status make_shape(const tahq_config *c, Shape *s)
{
    if (!c) return TAHQ_ERR_NULL;
    // shorter structs are the layouts from before alloc_tile (48 bytes) and low_bits (52 bytes) were added
    if (c->struct_size != sizeof(tahq_config) && c->struct_size != 48u && c->struct_size != 52u)
        return TAHQ_ERR_INVALID_ARG;
    const uint32_t A = (c->struct_size == 48u || c->alloc_tile == 0) ? c->tile : c->alloc_tile;
    const uint32_t low = (c->struct_size < 56u || c->low_bits == 0) ? 3u : c->low_bits;
    if (low < 1u || low > 7u) return TAHQ_ERR_INVALID_ARG;
    if (c->batch == 0 || c->seq == 0 || c->hidden == 0) return TAHQ_ERR_INVALID_ARG;
    if (c->tile == 0 || c->hidden % c->tile != 0) return TAHQ_ERR_INVALID_ARG;
    if (c->dtype > TAHQ_BF16 || c->scope > 1) return TAHQ_ERR_INVALID_ARG;
    if (!(c->budget_bits >= (float)low && c->budget_bits <= (float)(low + 1u))) return TAHQ_ERR_INVALID_ARG;
    if (A % c->tile != 0 || c->hidden % A != 0) return TAHQ_ERR_INVALID_ARG;
    if (c->tile != 8 && c->tile != 16 && c->tile != 32 && c->tile != 64 && c->tile != 128) return TAHQ_ERR_UNSUPPORTED;
    uint64_t M = c->hidden / c->tile;
    uint64_t T = (uint64_t)c->batch * c->seq * M;
    if (T >= (1ull << 31)) return TAHQ_ERR_UNSUPPORTED;
    s->B = c->batch; s->S = c->seq; s->C = c->hidden; s->G = c->tile;
    s->dtype = c->dtype; s->scope = c->scope;
    s->T = T;
    s->low = low;
    s->A = A;
    s->m = A / c->tile;
    s->n = c->scope ? T : (uint64_t)c->seq * M;
    s->U = c->scope ? 1u : c->batch;
    s->nA = s->n / s->m;
    double n = (double)s->nA;
    double k = __builtin_floor((double)c->budget_bits * n - (double)low * n + 0.5);
    if (k < 0) k = 0;
    if (k > n) k = n;
    s->kA = (uint64_t)k;
    s->k = s->kA * s->m;
    return TAHQ_OK;
}

void make_layout(const Shape &s, Layout *L)
{
    L->bitmap = 64;
    L->ranks = L->bitmap + pad64((s.T + 7) / 8);
    L->pivot = L->ranks + pad64(4 * ((s.T + 63) / 64));
    L->scale = L->pivot + pad64(s.T);
    L->zero = L->scale + pad64(2 * s.T);
    L->payload = L->zero + pad64(2 * s.T);
    L->total = L->payload + (uint64_t)(s.G / 8) * (s.low * s.T + (uint64_t)s.U * s.k);
}

void make_workspace(const Shape &s, Workspace *w)
{
    w->nseg = (uint32_t)((s.nA + kSegTiles - 1) / kSegTiles);
    uint64_t hb = (s.nA + kRadixKeysPerBlock - 1) / kRadixKeysPerBlock;
    w->hb = (uint32_t)(hb > 64 ? 64 : hb);
    uint64_t off = 0;
    w->hist0 = off;  off += (uint64_t)s.U * kDigit0Bins * 4;
    w->coarse = off; off += (uint64_t)s.U * 2 * 64 * 4;
    w->state = off;  off += (uint64_t)s.U * 8 * 4;
    w->lin_hist = off; off += (uint64_t)s.U * kLinBins * 4;
    w->fused = off;  off += (uint64_t)s.U * 4 * 4;
    w->zero_bytes = off;
    off = pad256(off);
    w->partial = off; off = pad256(off + (uint64_t)s.U * 2 * w->hb * kHistBins * 4);
    w->cand = off;  off = pad256(off + (uint64_t)s.U * kCandCap * 8);
    w->block_above = off; off = pad256(off + (uint64_t)s.U * ((s.nA + 16383) / 16384) * 4);
    w->keys = off;  off = pad256(off + s.T * 4);
    w->seg = off;   off = pad256(off + (uint64_t)s.U * w->nseg * 8);
    w->sel = off;   off = pad256(off + s.T);
    w->part = w->inv_norm = w->ranks_a = off;
    if (s.m > 1) {
        const uint64_t TA = s.T / s.m;
        w->part = off;     off = pad256(off + s.T * 4);
        w->inv_norm = off; off = pad256(off + TA * 4);
        w->ranks_a = off;  off = pad256(off + ((TA + 63) / 64) * 4);
    }
    w->total = off;
}

// -------------------------------------------------------------- device side

constexpr float kLn2 = 0x1.62e430p-1f;

// log(u), u > 0: frexp split, degree-5 Horner chain of fused multiply-adds on the
// mantissa in [0.5, 1), then e*ln2 added by one more fma.  |error| <= 1.1e-5.
__device__ __forceinline__ float log_contract(float u)
{
    float m = __builtin_amdgcn_frexp_mantf(u);
    int e = __builtin_amdgcn_frexp_expf(u);
    float P = 0x1.00ef0ap+0f;
    P = __builtin_fmaf(P, m, -0x1.29aa42p+2f);
    P = __builtin_fmaf(P, m, 0x1.22ea48p+3f);
    P = __builtin_fmaf(P, m, -0x1.3c1c5cp+3f);
    P = __builtin_fmaf(P, m, 0x1.c4859ep+2f);
    P = __builtin_fmaf(P, m, -0x1.5165a2p+1f);
    return __builtin_fmaf((float)e, kLn2, P);
}

// Order-preserving 32-bit key of an entropy (larger entropy -> larger key).
__device__ __forceinline__ uint32_t order_key(float h)
{
    const uint32_t u = __float_as_uint(h);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Linear bin of an entropy, 0 .. kLinBins - 1: non-decreasing in the entropy's order-preserving key (so a higher bin
// means a higher rank), and the same instruction sequence wherever it is evaluated.  Negative values go to bin 0; a NaN
// goes where its key goes: above +infinity with the sign bit clear, below -infinity with it set.
__device__ __forceinline__ uint32_t linear_bin(float h, float scale)
{
    // the median of three takes a NaN for the smallest of the three (bin 0, where a NaN with the sign bit set belongs)
    const uint32_t b = (uint32_t)__builtin_amdgcn_fmed3f(h * scale, 0.0f, (float)(kLinBins - 1));
    return (int32_t)__float_as_uint(h) > 0x7f800000 ? kLinBins - 1 : b;
}

// Sub-bin of an entropy that lies in linear bin `b`, 0 .. kSubBins - 1: non-decreasing in the entropy's key.  h * scale
// is the product linear_bin rounds down; its distance to b is exact in fp32, and so is the multiplication by a power of
// two.
__device__ __forceinline__ uint32_t linear_sub_bin(float h, float scale, uint32_t b)
{
    const uint32_t s = (uint32_t)__builtin_amdgcn_fmed3f((h * scale - (float)b) * (float)kSubBins, 0.0f, (float)(kSubBins - 1));
    return (int32_t)__float_as_uint(h) > 0x7f800000 ? kSubBins - 1 : s;
}

// The entropy an order-preserving key was made from.
__device__ __forceinline__ float key_to_float(uint32_t key)
{
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// fp32(1/sqrt(G)), the normalisation of Eq. 4.
template <int G> struct TileConst;
template <> struct TileConst<8>   { static constexpr float c = 0x1.6a09e6p-2f; };
template <> struct TileConst<16>  { static constexpr float c = 0.25f; };
template <> struct TileConst<32>  { static constexpr float c = 0x1.6a09e6p-3f; };
template <> struct TileConst<64>  { static constexpr float c = 0.125f; };
template <> struct TileConst<128> { static constexpr float c = 0x1.6a09e6p-4f; };

// ---- binary16 metadata, rounded outwards ---------------------------------

__device__ __forceinline__ float clamp_f16_range(float x)
{
    return __builtin_fminf(__builtin_fmaxf(x, -65504.0f), 65504.0f);
}
__device__ __forceinline__ uint32_t f16_bits(_Float16 h)
{
    return (uint32_t)__builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ float f16_widen(uint32_t bits)
{
    return (float)__builtin_bit_cast(_Float16, (unsigned short)bits);
}
// largest binary16 <= x
__device__ __forceinline__ uint32_t f16_down(float x)
{
    const float xc = clamp_f16_range(x);
    uint32_t h = f16_bits((_Float16)xc);                       // round to nearest even
    if (f16_widen(h) > xc)
        h = ((h & 0x7fffu) == 0) ? 0x8001u : ((h & 0x8000u) ? h + 1 : h - 1);
    return h == 0x8000u ? 0u : h;
}
// smallest binary16 >= x
__device__ __forceinline__ uint32_t f16_up(float x)
{
    const float xc = clamp_f16_range(x);
    uint32_t h = f16_bits((_Float16)xc);
    if (f16_widen(h) < xc)
        h = ((h & 0x7fffu) == 0) ? 0x0001u : ((h & 0x8000u) ? h - 1 : h + 1);
    return h == 0x8000u ? 0u : h;
}

}  // namespace tahq
