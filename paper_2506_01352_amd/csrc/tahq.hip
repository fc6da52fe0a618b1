// TAH-Quant stage-boundary activation codec for gfx950: kernels and C ABI.
//
// Paper sections implemented here: Sec. 3.1 (tiles of G contiguous channels),
// Sec. 3.2 Eq. 1-2 (entropy) and top-p% selection, Sec. 3.3 Eq. 3-4 (outlier
// test, pivot swap, Hadamard transform, asymmetric quantizer), Sec. 3.4 (byte
// stream), Alg. 1 step 5 (dequantize).
//
// Numerics contract (identical results on any mapping of tiles to lanes):
//   * all arithmetic is IEEE binary32, no contraction (-ffp-contract=off);
//     fused multiply-adds only where written (__builtin_fmaf);
//   * sums over a tile use the adjacent-pair binary tree;
//   * the Hadamard butterfly runs its stages h = 1, 2, ..., G/2 in that order;
//   * log(u) = e*ln2 + P(m) with (m, e) = frexp(u) and a fixed degree-5 polynomial;
//   * scale / zero-point are binary16, rounded outwards (up / down).
//
// Thread mapping of the streaming kernels: a lane holds 8 consecutive elements
// of a tile, L = G/8 neighbouring lanes hold one tile (L = 4, 8 or 16 lanes of
// one wavefront); reductions and the upper butterfly stages cross lanes.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "tahq.h"

namespace {

// ---------------------------------------------------------------- host side

struct Shape {
    uint32_t B, S, C, G, dtype, scope;
    uint64_t T;   // tiles in the tensor
    uint64_t n;   // tiles per ranking unit
    uint32_t U;   // ranking units
    uint64_t k;   // 4-bit tiles per ranking unit
};

struct Layout {
    uint64_t bitmap, ranks, pivot, scale, zero, payload, total;
};

constexpr uint32_t kSegTiles = 512;      // tiles one wavefront handles in the selection kernels
constexpr uint32_t kHistBins = 2048;

struct Workspace {
    // offsets in bytes from the workspace base
    uint64_t hist;       // uint32[U][3][kHistBins]           (zeroed per call)
    uint64_t done;       // uint32[U][4] tickets               (zeroed per call)
    uint64_t state;      // uint32[U][8] selection state
    uint64_t zero_bytes; // bytes from `hist` that must be zero before the selection starts
    uint64_t keys;       // float[T] entropies
    uint64_t seg;        // uint32[U][nseg][4]: eq, gt, eq_prefix, rank_base
    uint64_t sel;        // uint8[T] (only when n % 64 != 0)
    uint64_t total;
    uint32_t nseg;       // segments per ranking unit
};

inline uint64_t pad64(uint64_t x) { return (x + 63u) & ~uint64_t(63); }
inline uint64_t pad256(uint64_t x) { return (x + 255u) & ~uint64_t(255); }

tahq_status make_shape(const tahq_config *c, Shape *s)
{
    if (!c) return TAHQ_ERR_NULL;
    if (c->struct_size != sizeof(tahq_config)) return TAHQ_ERR_INVALID_ARG;
    if (c->batch == 0 || c->seq == 0 || c->hidden == 0) return TAHQ_ERR_INVALID_ARG;
    if (c->tile == 0 || c->hidden % c->tile != 0) return TAHQ_ERR_INVALID_ARG;
    if (c->dtype > TAHQ_BF16 || c->scope > 1) return TAHQ_ERR_INVALID_ARG;
    if (!(c->budget_bits >= 3.0f && c->budget_bits <= 4.0f)) return TAHQ_ERR_INVALID_ARG;
    if (c->tile != 32 && c->tile != 64 && c->tile != 128) return TAHQ_ERR_UNSUPPORTED;
    uint64_t M = c->hidden / c->tile;
    uint64_t T = (uint64_t)c->batch * c->seq * M;
    if (T >= (1ull << 31)) return TAHQ_ERR_UNSUPPORTED;
    s->B = c->batch; s->S = c->seq; s->C = c->hidden; s->G = c->tile;
    s->dtype = c->dtype; s->scope = c->scope;
    s->T = T;
    s->n = c->scope ? T : (uint64_t)c->seq * M;
    s->U = c->scope ? 1u : c->batch;
    double n = (double)s->n;
    double k = __builtin_floor((double)c->budget_bits * n - 3.0 * n + 0.5);
    if (k < 0) k = 0;
    if (k > n) k = n;
    s->k = (uint64_t)k;
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
    L->total = L->payload + (uint64_t)(s.G / 8) * (3 * s.T + (uint64_t)s.U * s.k);
}

void make_workspace(const Shape &s, Workspace *w)
{
    w->nseg = (uint32_t)((s.n + kSegTiles - 1) / kSegTiles);
    uint64_t off = 0;
    w->hist = off;  off += (uint64_t)s.U * 3 * kHistBins * 4;
    w->done = off;  off += (uint64_t)s.U * 4 * 4;
    w->state = off; off += (uint64_t)s.U * 8 * 4;
    w->zero_bytes = off;
    off = pad256(off);
    w->keys = off;  off = pad256(off + s.T * 4);
    w->seg = off;   off = pad256(off + (uint64_t)s.U * w->nseg * 16);
    w->sel = off;   off = pad256(off + s.T);
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

__device__ __forceinline__ float tree8(const float *z)
{
    return ((z[0] + z[1]) + (z[2] + z[3])) + ((z[4] + z[5]) + (z[6] + z[7]));
}

__device__ __forceinline__ float xor_lane(float v, int m) { return __shfl_xor(v, m, 64); }
__device__ __forceinline__ uint32_t xor_lane(uint32_t v, int m) { return (uint32_t)__shfl_xor((int)v, m, 64); }

// Sum over the L lanes of a tile, continuing the adjacent-pair tree across lanes.
template <int L>
__device__ __forceinline__ float tile_sum(float s)
{
#pragma unroll
    for (int m = 1; m < L; m <<= 1) s = s + xor_lane(s, m);
    return s;
}

template <bool BF16>
__device__ __forceinline__ void load8(const void *in, uint64_t elem, float *x)
{
    if constexpr (BF16) {
        const uint4 w = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(in) + elem);
        const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(ws[i] << 16);
            x[2 * i + 1] = __uint_as_float(ws[i] & 0xffff0000u);
        }
    } else {
        const float4 a = *reinterpret_cast<const float4 *>(static_cast<const float *>(in) + elem);
        const float4 b = *reinterpret_cast<const float4 *>(static_cast<const float *>(in) + elem + 4);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
}

// fp32 -> bf16 bits, round to nearest even (finite values).
__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <bool BF16>
__device__ __forceinline__ void store8(void *out, uint64_t elem, const float *x)
{
    if constexpr (BF16) {
        uint4 w;
        w.x = bf16_rne(x[0]) | (bf16_rne(x[1]) << 16);
        w.y = bf16_rne(x[2]) | (bf16_rne(x[3]) << 16);
        w.z = bf16_rne(x[4]) | (bf16_rne(x[5]) << 16);
        w.w = bf16_rne(x[6]) | (bf16_rne(x[7]) << 16);
        *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(out) + elem) = w;
    } else {
        float *o = static_cast<float *>(out) + elem;
        *reinterpret_cast<float4 *>(o) = make_float4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<float4 *>(o + 4) = make_float4(x[4], x[5], x[6], x[7]);
    }
}

// Eq. 1-2 for the tile spread over L lanes (8 raw elements per lane).
template <int L>
__device__ __forceinline__ float tile_entropy(const float *x, float eps_l1, float eps_log)
{
    float a[8], w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = __builtin_fabsf(x[i]);
    const float L1 = tile_sum<L>(tree8(a));
    const float invL = 1.0f / (L1 + eps_l1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float p = a[i] * invL;
        const float u = p + eps_log;
        w[i] = p * log_contract(u);
    }
    return 0.0f - tile_sum<L>(tree8(w));
}

// The unnormalised Sylvester butterfly over the tile: stages h = 1, 2, 4 inside the
// lane, stages h = 8 .. G/2 between lanes t and t ^ (h/8).
template <int L>
__device__ __forceinline__ void tile_butterfly(float *x, int t)
{
#pragma unroll
    for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if ((i & h) == 0) {
                const float p = x[i], q = x[i + h];
                x[i] = p + q;
                x[i + h] = p - q;
            }
        }
    }
#pragma unroll
    for (int m = 1; m < L; m <<= 1) {
        const bool upper = (t & m) != 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float other = xor_lane(x[i], m);
            x[i] = upper ? (other - x[i]) : (x[i] + other);
        }
    }
}

template <int G> struct TileConst;
template <> struct TileConst<32>  { static constexpr float c = 0x1.6a09e6p-3f; };
template <> struct TileConst<64>  { static constexpr float c = 0.125f; };
template <> struct TileConst<128> { static constexpr float c = 0x1.6a09e6p-4f; };

// Swap coordinates 0 and d of the tile held by L lanes (P_d of Sec. 3.3).
template <int L>
__device__ __forceinline__ void tile_swap(float *x, int t, int lane_base, uint32_t d)
{
    const float v0 = __shfl(x[0], lane_base, 64);
    float mine = x[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mine = ((d & 7u) == (uint32_t)i) ? x[i] : mine;
    const float vd = __shfl(mine, lane_base + (int)(d >> 3), 64);
    if (t == 0) x[0] = vd;
    const bool holder = (uint32_t)t == (d >> 3);
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (holder && (d & 7u) == (uint32_t)i) x[i] = v0;
}

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

// -------------------------------------------------------------- K0: entropy

template <int G, bool BF16>
__global__ __launch_bounds__(256) void k_entropy(const void *__restrict__ in, float *__restrict__ H,
                                                 uint32_t T, float eps_l1, float eps_log)
{
    constexpr int L = G / 8;
    const uint64_t gid = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t j = gid / L;
    const int t = (int)(gid % L);
    // lanes of a tile leave together: T*L is a multiple of L
    if (j >= T) return;
    float x[8];
    load8<BF16>(in, j * G + (uint64_t)t * 8, x);
    const float h = tile_entropy<L>(x, eps_l1, eps_log);
    if (t == 0) H[j] = h;
}

// ------------------------------------------------- K2: top-k by radix select

__device__ __forceinline__ uint32_t order_key(float h)
{
    const uint32_t u = __float_as_uint(h);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint32_t agent_load(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Exclusive scan of one value per thread over a block of 256 threads.
__device__ __forceinline__ uint32_t block_scan_256(uint32_t v, uint32_t *lds /*[256]*/, uint32_t *total)
{
    const int tid = threadIdx.x;
    lds[tid] = v;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        uint32_t add = (tid >= off) ? lds[tid - off] : 0u;
        __syncthreads();
        lds[tid] += add;
        __syncthreads();
    }
    const uint32_t incl = lds[tid];
    *total = lds[255];
    __syncthreads();
    return incl - v;
}

// selection state of one ranking unit (uint32[8] in the workspace)
enum { ST_BIN0 = 0, ST_BIN1 = 1, ST_BIN2 = 2, ST_KREM = 3, ST_KEY = 4, ST_TAKE = 5 };

// One radix pass: histogram of the digit `pass` of the keys whose higher digits match
// the bins already chosen; the last block of each unit to finish picks the bin that
// holds the k-th largest key and how many keys are still wanted inside it.
// Digits: pass 0 = bits 31..21, pass 1 = bits 20..10, pass 2 = bits 9..0.
__global__ __launch_bounds__(256) void k_radix_pass(const float *__restrict__ H, uint32_t n, uint32_t k,
                                                    int pass, uint32_t *hist, uint32_t *done,
                                                    uint32_t *state)
{
    __shared__ uint32_t lh[kHistBins];
    __shared__ uint32_t scan[256];
    __shared__ uint32_t ticket;
    const uint32_t u = blockIdx.y;
    const int tid = threadIdx.x;
    uint32_t *uh = hist + ((uint64_t)u * 3 + pass) * kHistBins;
    uint32_t *ust = state + (uint64_t)u * 8;
    const float *uH = H + (uint64_t)u * n;

    for (int i = tid; i < (int)kHistBins; i += 256) lh[i] = 0;
    __syncthreads();

    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const uint32_t mask = pass == 2 ? 1023u : 2047u;
    uint32_t want_hi = 0;
    int hi_shift = 32;   // compare key >> hi_shift with want_hi (pass 0: nothing to compare)
    if (pass == 1) { want_hi = ust[ST_BIN0]; hi_shift = 21; }
    if (pass == 2) { want_hi = (ust[ST_BIN0] << 11) | ust[ST_BIN1]; hi_shift = 10; }

    for (uint64_t i = (uint64_t)blockIdx.x * 256 + tid; i < n; i += (uint64_t)gridDim.x * 256) {
        const uint32_t key = order_key(uH[i]);
        const bool match = (pass == 0) || ((key >> hi_shift) == want_hi);
        if (match) atomicAdd(&lh[(key >> shift) & mask], 1u);
    }
    __syncthreads();
    for (int i = tid; i < (int)kHistBins; i += 256)
        if (lh[i]) atomicAdd(&uh[i], lh[i]);
    __threadfence();
    __syncthreads();
    if (tid == 0) ticket = atomicAdd(&done[(uint64_t)u * 4 + pass], 1u);
    __syncthreads();
    if (ticket != gridDim.x - 1) return;
    __threadfence();

    // Last block of this unit: walk the bins from the top.  Thread t owns the 8 bins
    // 2047-8t .. 2040-8t (descending), so prefix sums run from the largest digit down.
    const uint32_t want = (pass == 0) ? k : ust[ST_KREM];
    uint32_t c[8], mine = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { c[i] = agent_load(&uh[kHistBins - 1 - (tid * 8 + i)]); mine += c[i]; }
    uint32_t total;
    uint32_t above = block_scan_256(mine, scan, &total);   // keys in bins above my 8 bins
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // the k-th largest lies in the bin where the running count first reaches `want`
        if (above < want && want <= above + c[i]) {
            ust[ST_BIN0 + pass] = kHistBins - 1 - (tid * 8 + i);
            ust[ST_KREM] = want - above;
            if (pass == 2) {
                ust[ST_KEY] = (ust[ST_BIN0] << 21) | (ust[ST_BIN1] << 10) | (kHistBins - 1 - (tid * 8 + i));
                ust[ST_TAKE] = want - above;
            }
        }
        above += c[i];
    }
}

// Per segment of 512 tiles (one wavefront): how many keys equal the threshold key and
// how many exceed it.  The last block of the unit turns these into exclusive prefixes:
// seg[.][2] = equal keys before the segment, seg[.][3] = 4-bit tiles before the segment
// in the whole tensor (every earlier unit contributes exactly k).
__global__ __launch_bounds__(256) void k_seg_count(const float *__restrict__ H, uint32_t n, uint32_t k,
                                                   uint32_t nseg, const uint32_t *__restrict__ state,
                                                   uint32_t *seg, uint32_t *done)
{
    __shared__ uint32_t scan[256];
    __shared__ uint32_t ticket;
    const uint32_t u = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t *ust = state + (uint64_t)u * 8;
    const uint32_t thr = ust[ST_KEY], take = ust[ST_TAKE];
    const float *uH = H + (uint64_t)u * n;
    uint32_t *useg = seg + (uint64_t)u * nseg * 4;

    const uint32_t s = blockIdx.x * 4 + wave;
    if (s < nseg) {
        uint32_t eq = 0, gt = 0;
        for (int r = 0; r < (int)(kSegTiles / 64); ++r) {
            const uint64_t j = (uint64_t)s * kSegTiles + r * 64 + lane;
            const bool valid = j < n;
            const uint32_t key = valid ? order_key(uH[j]) : 0u;
            eq += __popcll(__ballot(valid && key == thr));
            gt += __popcll(__ballot(valid && key > thr));
        }
        if (lane == 0) { useg[(uint64_t)s * 4 + 0] = eq; useg[(uint64_t)s * 4 + 1] = gt; }
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) ticket = atomicAdd(&done[(uint64_t)u * 4 + 3], 1u);
    __syncthreads();
    if (ticket != gridDim.x - 1) return;
    __threadfence();

    uint32_t eq_carry = 0, rank_carry = u * k;
    for (uint32_t base = 0; base < nseg; base += 256) {
        const uint32_t i = base + tid;
        const uint32_t eq = (i < nseg) ? agent_load(&useg[(uint64_t)i * 4 + 0]) : 0u;
        const uint32_t gt = (i < nseg) ? agent_load(&useg[(uint64_t)i * 4 + 1]) : 0u;
        uint32_t eq_total, sel_total;
        const uint32_t eq_before = eq_carry + block_scan_256(eq, scan, &eq_total);
        // equal keys are taken in index order until `take` of them are used up
        const uint32_t left = eq_before < take ? take - eq_before : 0u;
        const uint32_t sel = gt + (eq < left ? eq : left);
        const uint32_t rank_before = rank_carry + block_scan_256(sel, scan, &sel_total);
        if (i < nseg) { useg[(uint64_t)i * 4 + 2] = eq_before; useg[(uint64_t)i * 4 + 3] = rank_before; }
        eq_carry += eq_total;
        rank_carry += sel_total;
    }
}

// Width bit of every tile, rank-table entries, and the bit map itself when units start on
// 64-tile boundaries (otherwise one byte per tile goes to `sel` and k_bitmap_pack follows).
__global__ __launch_bounds__(256) void k_assign(const float *__restrict__ H, uint32_t n, uint32_t nseg,
                                                const uint32_t *__restrict__ state,
                                                const uint32_t *__restrict__ seg,
                                                uint64_t *__restrict__ bitmap, uint32_t *__restrict__ ranks,
                                                uint8_t *__restrict__ sel_bytes, int aligned)
{
    const uint32_t u = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t s = blockIdx.x * 4 + wave;
    if (s >= nseg) return;
    const uint32_t *ust = state + (uint64_t)u * 8;
    const uint32_t thr = ust[ST_KEY], take = ust[ST_TAKE];
    const float *uH = H + (uint64_t)u * n;
    const uint32_t *sg = seg + ((uint64_t)u * nseg + s) * 4;
    uint32_t eq_run = sg[2], rank_run = sg[3];
    const uint64_t below = (1ull << lane) - 1ull;
    for (int r = 0; r < (int)(kSegTiles / 64); ++r) {
        const uint64_t jl = (uint64_t)s * kSegTiles + r * 64 + lane;
        const bool valid = jl < n;
        const uint32_t key = valid ? order_key(uH[jl]) : 0u;
        const bool eq = valid && key == thr;
        const uint64_t eq_mask = __ballot(eq);
        const bool sel = valid && (key > thr || (eq && eq_run + __popcll(eq_mask & below) < take));
        const uint64_t sel_mask = __ballot(sel);
        const uint64_t jg = (uint64_t)u * n + jl;     // tile index in the tensor
        if (aligned) {
            if (lane == 0 && valid) { bitmap[jg >> 6] = sel_mask; ranks[jg >> 6] = rank_run; }
        } else if (valid) {
            sel_bytes[jg] = sel ? 1 : 0;
            if ((jg & 63u) == 0) ranks[jg >> 6] = rank_run + __popcll(sel_mask & below);
        }
        eq_run += __popcll(eq_mask);
        rank_run += __popcll(sel_mask);
    }
}

__global__ __launch_bounds__(256) void k_bitmap_pack(const uint8_t *__restrict__ sel_bytes, uint32_t T,
                                                     uint64_t *__restrict__ bitmap)
{
    const uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t word = __ballot(j < T && sel_bytes[j < T ? j : 0] != 0);
    if ((threadIdx.x & 63) == 0 && (j >> 6) < ((uint64_t)T + 63) / 64) bitmap[j >> 6] = word;
}

// Budget 3.0 or 4.0: every tile has the same width.
__global__ __launch_bounds__(256) void k_bitmap_const(uint32_t T, int all4, uint64_t *__restrict__ bitmap,
                                                      uint32_t *__restrict__ ranks)
{
    const uint64_t w = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t words = ((uint64_t)T + 63) / 64;
    if (w >= words) return;
    uint64_t bits = 0;
    if (all4) {
        const uint64_t left = (uint64_t)T - w * 64;
        bits = left >= 64 ? ~0ull : ((1ull << left) - 1ull);
    }
    bitmap[w] = bits;
    ranks[w] = all4 ? (uint32_t)(w * 64) : 0u;
}

// Header, zeroed section padding, zeroed selection scratch.
struct HeaderWords { uint32_t w[16]; };
struct PadList { uint64_t begin[5]; uint32_t len[5]; };

__global__ __launch_bounds__(256) void k_prologue(uint8_t *__restrict__ packed, HeaderWords hdr, PadList pads,
                                                  uint32_t *__restrict__ zero_base, uint32_t zero_words)
{
    const uint32_t gid = blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0) {
        if (threadIdx.x < 16) reinterpret_cast<uint32_t *>(packed)[threadIdx.x] = hdr.w[threadIdx.x];
        for (int s = 0; s < 5; ++s)
            if (threadIdx.x < pads.len[s]) packed[pads.begin[s] + threadIdx.x] = 0;
    }
    for (uint32_t i = gid; i < zero_words; i += gridDim.x * 256) zero_base[i] = 0u;
}

// ------------------------------------ K3: transform + quantize + pack

template <int G, bool BF16>
__global__ __launch_bounds__(256) void k_quant_pack(const void *__restrict__ in, uint8_t *__restrict__ packed,
                                                    Layout lay, uint32_t T, float tau, float eps_ratio)
{
    constexpr int L = G / 8;
    const uint64_t gid = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t j = gid / L;
    const int t = (int)(gid % L);
    if (j >= T) return;
    const int lane = threadIdx.x & 63;
    const int lane_base = lane - t;

    float x[8];
    load8<BF16>(in, j * G + (uint64_t)t * 8, x);

    // Eq. 3: largest and second-largest magnitude (with multiplicity), pivot = lowest index of the largest
    float a1 = __builtin_fabsf(x[0]), a2 = 0.0f;
    uint32_t k1 = (uint32_t)t * 8;
#pragma unroll
    for (int i = 1; i < 8; ++i) {
        const float a = __builtin_fabsf(x[i]);
        const bool gt = a > a1;
        a2 = gt ? a1 : __builtin_fmaxf(a2, a);
        k1 = gt ? (uint32_t)t * 8 + i : k1;
        a1 = gt ? a : a1;
    }
#pragma unroll
    for (int m = 1; m < L; m <<= 1) {
        const float b1 = xor_lane(a1, m), b2 = xor_lane(a2, m);
        const uint32_t kb = xor_lane(k1, m);
        const bool take_b = b1 > a1 || (b1 == a1 && kb < k1);
        a2 = __builtin_fmaxf(__builtin_fminf(a1, b1), __builtin_fmaxf(a2, b2));
        a1 = __builtin_fmaxf(a1, b1);
        k1 = take_b ? kb : k1;
    }
    const float thr = tau * (a2 + eps_ratio);
    const bool flag = a1 > thr;
    const uint32_t d = k1;

    // Eq. 4 on outlier tiles
    if (flag) {
        tile_swap<L>(x, t, lane_base, d);
        tile_butterfly<L>(x, t);
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = x[i] * TileConst<G>::c;
    }

    float mn = x[0], mx = x[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) { mn = __builtin_fminf(mn, x[i]); mx = __builtin_fmaxf(mx, x[i]); }
#pragma unroll
    for (int m = 1; m < L; m <<= 1) {
        mn = __builtin_fminf(mn, xor_lane(mn, m));
        mx = __builtin_fmaxf(mx, xor_lane(mx, m));
    }
    mn = mn + 0.0f;
    mx = mx + 0.0f;

    // width and payload position from the bit map and the rank table
    const uint64_t word = reinterpret_cast<const uint64_t *>(packed + lay.bitmap)[j >> 6];
    const uint32_t bit = (uint32_t)(j & 63u);
    const uint32_t b = 3u + (uint32_t)((word >> bit) & 1ull);
    const uint32_t rank = reinterpret_cast<const uint32_t *>(packed + lay.ranks)[j >> 6] +
                          (uint32_t)__popcll(word & ((1ull << bit) - 1ull));

    // asymmetric quantizer, binary16 metadata rounded outwards
    const float Lv = (b == 4u) ? 15.0f : 7.0f;
    const uint32_t z16 = f16_down(mn);
    const float mnf = f16_widen(z16);
    const float s = (mx - mnf) / Lv;
    uint32_t s16 = f16_up(s);
    if ((s16 & 0x7fffu) == 0) s16 = 0x3c00u;
    const float sf = f16_widen(s16);
    const float rcp = 1.0f / sf;

    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float q = __builtin_fminf(__builtin_fmaxf(__builtin_rintf((x[i] - mnf) * rcp), 0.0f), Lv);
        w |= (uint32_t)q << (b * i);
    }

    uint32_t *pay = reinterpret_cast<uint32_t *>(packed + lay.payload) + (uint64_t)(G / 32) * (3ull * j + rank);
    // three-bit tiles: four lanes' 24-bit strings make three dwords
    const uint32_t nxt = (uint32_t)__shfl((int)w, lane + 1, 64);
    if (b == 4u) {
        pay[t] = w;
    } else {
        const int r4 = t & 3;
        if (r4 < 3) pay[3 * (t >> 2) + r4] = (w >> (8 * r4)) | (nxt << (24 - 8 * r4));
    }
    if (t == 0) {
        reinterpret_cast<uint16_t *>(packed + lay.scale)[j] = (uint16_t)s16;
        reinterpret_cast<uint16_t *>(packed + lay.zero)[j] = (uint16_t)z16;
        packed[lay.pivot + j] = flag ? (uint8_t)(0x80u | d) : (uint8_t)0;
    }
}

// ------------------------------------------------------------- K4: decode

template <int G, bool OUT_BF16>
__global__ __launch_bounds__(256) void k_decode(const uint8_t *__restrict__ packed, void *__restrict__ out,
                                                Layout lay, uint32_t T)
{
    constexpr int L = G / 8;
    const uint64_t gid = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t j = gid / L;
    const int t = (int)(gid % L);
    if (j >= T) return;
    const int lane = threadIdx.x & 63;
    const int lane_base = lane - t;

    const uint64_t word = reinterpret_cast<const uint64_t *>(packed + lay.bitmap)[j >> 6];
    const uint32_t bit = (uint32_t)(j & 63u);
    const uint32_t b = 3u + (uint32_t)((word >> bit) & 1ull);
    const uint32_t rank = reinterpret_cast<const uint32_t *>(packed + lay.ranks)[j >> 6] +
                          (uint32_t)__popcll(word & ((1ull << bit) - 1ull));
    const uint32_t s16 = reinterpret_cast<const uint16_t *>(packed + lay.scale)[j];
    const uint32_t z16 = reinterpret_cast<const uint16_t *>(packed + lay.zero)[j];
    const uint32_t pv = packed[lay.pivot + j];
    const float sf = f16_widen(s16), mnf = f16_widen(z16);

    const uint32_t *pay = reinterpret_cast<const uint32_t *>(packed + lay.payload) + (uint64_t)(G / 32) * (3ull * j + rank);
    uint32_t w;
    if (b == 4u) {
        w = pay[t];
    } else {
        // my 24 bits start at byte 3t: inside the group of three dwords that four lanes share
        const int r4 = t & 3;
        const uint32_t *grp = pay + 3 * (t >> 2);
        const int di = (3 * r4) >> 2;            // 0, 0, 1, 2
        const int sh = 8 * ((3 * r4) & 3);       // 0, 24, 16, 8
        const uint32_t lo = grp[di];
        const uint32_t hi = grp[di < 2 ? di + 1 : 2];
        w = sh == 0 ? lo : ((lo >> sh) | (hi << (32 - sh)));
        w &= 0x00ffffffu;
    }

    float x[8];
    const uint32_t cmask = (1u << b) - 1u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t q = (w >> (b * i)) & cmask;
        x[i] = __builtin_fmaf((float)q, sf, mnf);
    }
    if (pv & 0x80u) {
        tile_butterfly<L>(x, t);
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = x[i] * TileConst<G>::c;
        tile_swap<L>(x, t, lane_base, pv & 0x7fu);
    }
    store8<OUT_BF16>(out, j * G + (uint64_t)t * 8, x);
}

// ------------------------------------------------------------ launch glue

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline uint32_t blocks_for(uint64_t threads) { return (uint32_t)((threads + 255) / 256); }

template <typename F32K, typename BF16K>
inline void pick(uint32_t dtype, F32K f, BF16K g) { if (dtype == TAHQ_BF16) g(); else f(); }

#define TAHQ_LAUNCH_G(KERNEL, G_, FLAG, grid, stream, ...)                                           \
    do {                                                                                             \
        if ((G_) == 32) {                                                                            \
            if (FLAG) hipLaunchKernelGGL((KERNEL<32, true>), grid, dim3(256), 0, stream, __VA_ARGS__);  \
            else hipLaunchKernelGGL((KERNEL<32, false>), grid, dim3(256), 0, stream, __VA_ARGS__);      \
        } else if ((G_) == 64) {                                                                     \
            if (FLAG) hipLaunchKernelGGL((KERNEL<64, true>), grid, dim3(256), 0, stream, __VA_ARGS__);  \
            else hipLaunchKernelGGL((KERNEL<64, false>), grid, dim3(256), 0, stream, __VA_ARGS__);      \
        } else {                                                                                     \
            if (FLAG) hipLaunchKernelGGL((KERNEL<128, true>), grid, dim3(256), 0, stream, __VA_ARGS__); \
            else hipLaunchKernelGGL((KERNEL<128, false>), grid, dim3(256), 0, stream, __VA_ARGS__);     \
        }                                                                                            \
    } while (0)

void launch_entropy(const Shape &s, const tahq_config *cfg, const void *d_in, float *d_H, hipStream_t st)
{
    const uint32_t grid = blocks_for(s.T * (s.G / 8));
    TAHQ_LAUNCH_G(k_entropy, s.G, s.dtype == TAHQ_BF16, dim3(grid), st, d_in, d_H, (uint32_t)s.T,
                  cfg->eps_l1, cfg->eps_log);
}

}  // namespace

// ------------------------------------------------------------------ C ABI

extern "C" {

void tahq_config_default(tahq_config *cfg)
{
    if (!cfg) return;
    memset(cfg, 0, sizeof *cfg);
    cfg->struct_size = (uint32_t)sizeof *cfg;
    cfg->tile = 64;
    cfg->dtype = TAHQ_BF16;
    cfg->scope = 0;
    cfg->budget_bits = 3.8f;
    cfg->tau = 2.0f;
    cfg->eps_l1 = 1e-8f;
    cfg->eps_log = 1e-8f;
    cfg->eps_ratio = 1e-8f;
}

uint64_t tahq_k_per_unit(const tahq_config *cfg)
{
    Shape s;
    if (make_shape(cfg, &s) != TAHQ_OK) return 0;
    return s.k;
}

size_t tahq_packed_size(const tahq_config *cfg)
{
    Shape s;
    if (make_shape(cfg, &s) != TAHQ_OK) return 0;
    Layout L;
    make_layout(s, &L);
    return (size_t)L.total;
}

size_t tahq_workspace_size(const tahq_config *cfg)
{
    Shape s;
    if (make_shape(cfg, &s) != TAHQ_OK) return 0;
    Workspace w;
    make_workspace(s, &w);
    return (size_t)w.total;
}

tahq_status tahq_tile_entropy(const tahq_config *cfg, const void *d_in, float *d_entropy, tahq_stream stream)
{
    Shape s;
    tahq_status rc = make_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    if (!d_in || !d_entropy) return TAHQ_ERR_NULL;
    if (misaligned(d_in) || misaligned(d_entropy)) return TAHQ_ERR_MISALIGNED;
    launch_entropy(s, cfg, d_in, d_entropy, (hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? TAHQ_OK : TAHQ_ERR_HIP;
}

tahq_status tahq_encode_phases(const tahq_config *cfg, const void *d_in, void *d_packed, size_t packed_capacity,
                               void *d_workspace, size_t workspace_capacity, uint32_t phases, tahq_stream stream)
{
    if (phases == 0 || (phases & ~(uint32_t)TAHQ_PHASE_ALL)) return TAHQ_ERR_INVALID_ARG;
    Shape s;
    tahq_status rc = make_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    if (!d_in || !d_packed || !d_workspace) return TAHQ_ERR_NULL;
    Layout lay;
    make_layout(s, &lay);
    Workspace ws;
    make_workspace(s, &ws);
    if (packed_capacity < lay.total) return TAHQ_ERR_BUFFER_TOO_SMALL;
    if (workspace_capacity < ws.total) return TAHQ_ERR_WORKSPACE_TOO_SMALL;
    if (misaligned(d_in) || misaligned(d_packed) || misaligned(d_workspace)) return TAHQ_ERR_MISALIGNED;

    hipStream_t st = (hipStream_t)stream;
    uint8_t *packed = static_cast<uint8_t *>(d_packed);
    uint8_t *wsb = static_cast<uint8_t *>(d_workspace);
    uint64_t *bitmap = reinterpret_cast<uint64_t *>(packed + lay.bitmap);
    uint32_t *ranks = reinterpret_cast<uint32_t *>(packed + lay.ranks);
    const bool select = s.k != 0 && s.k != s.n;

    // header, section padding, selection scratch
    HeaderWords hdr;
    memset(&hdr, 0, sizeof hdr);
    hdr.w[0] = 0x51484154u;   // "TAHQ"
    hdr.w[1] = 1;
    hdr.w[2] = s.dtype; hdr.w[3] = s.B; hdr.w[4] = s.S; hdr.w[5] = s.C; hdr.w[6] = s.G; hdr.w[7] = s.scope;
    hdr.w[8] = (uint32_t)s.k;
    memcpy(&hdr.w[9], &cfg->budget_bits, 4);
    memcpy(&hdr.w[10], &cfg->tau, 4);
    memcpy(&hdr.w[11], &cfg->eps_l1, 4);
    memcpy(&hdr.w[12], &cfg->eps_log, 4);
    memcpy(&hdr.w[13], &cfg->eps_ratio, 4);
    PadList pads;
    const uint64_t words64 = (s.T + 63) / 64;
    const uint64_t sec_begin[5] = {lay.bitmap + words64 * 8, lay.ranks + words64 * 4, lay.pivot + s.T,
                                   lay.scale + 2 * s.T, lay.zero + 2 * s.T};
    const uint64_t sec_end[5] = {lay.ranks, lay.pivot, lay.scale, lay.zero, lay.payload};
    for (int i = 0; i < 5; ++i) { pads.begin[i] = sec_begin[i]; pads.len[i] = (uint32_t)(sec_end[i] - sec_begin[i]); }
    const uint32_t zero_words = select ? (uint32_t)(ws.zero_bytes / 4) : 0u;
    if (phases & TAHQ_PHASE_PROLOGUE)
        hipLaunchKernelGGL(k_prologue, dim3(select ? 64 : 1), dim3(256), 0, st, packed, hdr, pads,
                           reinterpret_cast<uint32_t *>(wsb + ws.hist), zero_words);

    if (select) {
        float *H = reinterpret_cast<float *>(wsb + ws.keys);
        uint32_t *hist = reinterpret_cast<uint32_t *>(wsb + ws.hist);
        uint32_t *done = reinterpret_cast<uint32_t *>(wsb + ws.done);
        uint32_t *state = reinterpret_cast<uint32_t *>(wsb + ws.state);
        uint32_t *seg = reinterpret_cast<uint32_t *>(wsb + ws.seg);
        uint8_t *sel = wsb + ws.sel;
        if (phases & TAHQ_PHASE_ENTROPY) launch_entropy(s, cfg, d_in, H, st);
        uint32_t hb = (uint32_t)((s.n + 256 * 16 - 1) / (256 * 16));
        if (hb > 1024) hb = 1024;
        for (int pass = 0; pass < 3 && (phases & TAHQ_PHASE_SELECT); ++pass)
            hipLaunchKernelGGL(k_radix_pass, dim3(hb, s.U), dim3(256), 0, st, (const float *)H, (uint32_t)s.n,
                               (uint32_t)s.k, pass, hist, done, state);
        const uint32_t sb = (ws.nseg + 3) / 4;
        if (phases & TAHQ_PHASE_SELECT) {
        hipLaunchKernelGGL(k_seg_count, dim3(sb, s.U), dim3(256), 0, st, (const float *)H, (uint32_t)s.n,
                           (uint32_t)s.k, ws.nseg, (const uint32_t *)state, seg, done);
        const int aligned = (s.n % 64 == 0) ? 1 : 0;
        hipLaunchKernelGGL(k_assign, dim3(sb, s.U), dim3(256), 0, st, (const float *)H, (uint32_t)s.n, ws.nseg,
                           (const uint32_t *)state, (const uint32_t *)seg, bitmap, ranks, sel, aligned);
        if (!aligned)
            hipLaunchKernelGGL(k_bitmap_pack, dim3(blocks_for(words64 * 64)), dim3(256), 0, st,
                               (const uint8_t *)sel, (uint32_t)s.T, bitmap);
        }
    } else if (phases & TAHQ_PHASE_SELECT) {
        hipLaunchKernelGGL(k_bitmap_const, dim3(blocks_for(words64)), dim3(256), 0, st, (uint32_t)s.T,
                           s.k == s.n ? 1 : 0, bitmap, ranks);
    }

    if (phases & TAHQ_PHASE_QUANT) {
        const uint32_t grid = blocks_for(s.T * (s.G / 8));
        TAHQ_LAUNCH_G(k_quant_pack, s.G, s.dtype == TAHQ_BF16, dim3(grid), st, d_in, packed, lay, (uint32_t)s.T,
                      cfg->tau, cfg->eps_ratio);
    }
    return hipGetLastError() == hipSuccess ? TAHQ_OK : TAHQ_ERR_HIP;
}

tahq_status tahq_encode(const tahq_config *cfg, const void *d_in, void *d_packed, size_t packed_capacity,
                        void *d_workspace, size_t workspace_capacity, tahq_stream stream)
{
    return tahq_encode_phases(cfg, d_in, d_packed, packed_capacity, d_workspace, workspace_capacity,
                              TAHQ_PHASE_ALL, stream);
}

tahq_status tahq_decode(const tahq_config *cfg, const void *d_packed, size_t packed_bytes, void *d_out,
                        uint32_t out_dtype, void *d_workspace, size_t workspace_capacity, tahq_stream stream)
{
    (void)d_workspace;
    (void)workspace_capacity;
    Shape s;
    tahq_status rc = make_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    if (out_dtype > TAHQ_BF16) return TAHQ_ERR_INVALID_ARG;
    if (!d_packed || !d_out) return TAHQ_ERR_NULL;
    Layout lay;
    make_layout(s, &lay);
    if (packed_bytes < lay.total) return TAHQ_ERR_BUFFER_TOO_SMALL;
    if (misaligned(d_packed) || misaligned(d_out)) return TAHQ_ERR_MISALIGNED;
    const uint32_t grid = blocks_for(s.T * (s.G / 8));
    hipStream_t st = (hipStream_t)stream;
    TAHQ_LAUNCH_G(k_decode, s.G, out_dtype == TAHQ_BF16, dim3(grid), st, static_cast<const uint8_t *>(d_packed),
                  d_out, lay, (uint32_t)s.T);
    return hipGetLastError() == hipSuccess ? TAHQ_OK : TAHQ_ERR_HIP;
}

tahq_status tahq_parse_header(const void *header64, tahq_config *cfg)
{
    if (!header64 || !cfg) return TAHQ_ERR_NULL;
    uint32_t w[16];
    memcpy(w, header64, 64);
    if (w[0] != 0x51484154u || w[1] != 1u) return TAHQ_ERR_INVALID_ARG;
    tahq_config_default(cfg);
    cfg->dtype = w[2]; cfg->batch = w[3]; cfg->seq = w[4]; cfg->hidden = w[5]; cfg->tile = w[6]; cfg->scope = w[7];
    memcpy(&cfg->budget_bits, &w[9], 4);
    memcpy(&cfg->tau, &w[10], 4);
    memcpy(&cfg->eps_l1, &w[11], 4);
    memcpy(&cfg->eps_log, &w[12], 4);
    memcpy(&cfg->eps_ratio, &w[13], 4);
    Shape s;
    tahq_status rc = make_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    return s.k == w[8] ? TAHQ_OK : TAHQ_ERR_INVALID_ARG;
}

const char *tahq_status_string(tahq_status s)
{
    switch (s) {
    case TAHQ_OK: return "ok";
    case TAHQ_ERR_NULL: return "a required pointer is NULL";
    case TAHQ_ERR_INVALID_ARG: return "invalid argument";
    case TAHQ_ERR_UNSUPPORTED: return "unsupported tile width or tensor too large";
    case TAHQ_ERR_BUFFER_TOO_SMALL: return "packed buffer too small";
    case TAHQ_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case TAHQ_ERR_MISALIGNED: return "device pointer not 16-byte aligned";
    case TAHQ_ERR_HIP: return "kernel launch failed";
    }
    return "unknown status";
}

uint32_t tahq_version(void) { return (1u << 16) | 0u; }

}  // extern "C"
