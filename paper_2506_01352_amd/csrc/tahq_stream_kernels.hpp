// Streaming kernels: entropy (Eq. 1-2), transform + quantize + pack (Eq. 3-4, Sec. 3.4),
// decode (Alg. 1 step 5).
//
// Mapping: ONE LANE OWNS ONE TILE.  The codec is bound by vector-ALU issue as much as by HBM, so the
// per-tile work (reductions, butterflies, quantizer parameters) is kept free of cross-lane traffic
// and of lane-redundant scalar work: a workgroup stages TILES consecutive tiles through LDS with
// coalesced 128-bit global accesses, then every lane pulls its whole tile into registers.  LDS rows
// are padded by 16 bytes so that the lane-per-row 128-bit reads are bank-conflict free.
#pragma once
#include "tahq_common.hpp"

namespace tahq {

// Geometry of one workgroup's batch of tiles for an element type of ESIZE bytes.
template <int G, int ESIZE>
struct Batch {
    static constexpr int BYTES = G * ESIZE;                                   // one tile
    static constexpr int TILES = (32768 / BYTES) < 256 ? (32768 / BYTES) : 256;   // tiles = threads per workgroup
    static constexpr int STRIDE = BYTES + 16;                                 // padded LDS row
    static constexpr int CHUNKS = BYTES / 16;                                 // 16-byte chunks per tile
    static constexpr int LDS_BYTES = TILES * STRIDE;
};

// Coalesced copy of `nvalid` tiles from global memory into padded LDS rows.
template <int G, int ESIZE>
__device__ __forceinline__ void stage_in(const void *__restrict__ in, uint64_t j0, uint32_t nvalid, uint8_t *lds)
{
    using B = Batch<G, ESIZE>;
    constexpr int UNR = B::CHUNKS < 8 ? B::CHUNKS : 8;
    const uint8_t *src = static_cast<const uint8_t *>(in) + j0 * B::BYTES;
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < B::CHUNKS; i += UNR) {
        uint4 v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t q = (uint32_t)(i + u) * B::TILES + tid;
            v[u] = make_uint4(0u, 0u, 0u, 0u);
            if (q / B::CHUNKS < nvalid) v[u] = *reinterpret_cast<const uint4 *>(src + (uint64_t)q * 16);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t q = (uint32_t)(i + u) * B::TILES + tid;
            const uint32_t tile = q / B::CHUNKS, sub = q % B::CHUNKS;
            if (tile < nvalid) *reinterpret_cast<uint4 *>(lds + tile * B::STRIDE + sub * 16) = v[u];
        }
    }
}

// Coalesced copy of `nvalid` tiles from padded LDS rows to global memory.
template <int G, int ESIZE>
__device__ __forceinline__ void stage_out(void *__restrict__ out, uint64_t j0, uint32_t nvalid, const uint8_t *lds)
{
    using B = Batch<G, ESIZE>;
    uint8_t *dst = static_cast<uint8_t *>(out) + j0 * B::BYTES;
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < B::CHUNKS; ++i) {
        const uint32_t q = (uint32_t)i * B::TILES + tid;
        const uint32_t tile = q / B::CHUNKS, sub = q % B::CHUNKS;
        if (tile < nvalid)
            *reinterpret_cast<uint4 *>(dst + (uint64_t)q * 16) = *reinterpret_cast<const uint4 *>(lds + tile * B::STRIDE + sub * 16);
    }
}

// My tile, from its LDS row into registers, widened to fp32.
template <int G, bool BF16>
__device__ __forceinline__ void read_tile(const uint8_t *row, float *x)
{
    if constexpr (BF16) {
#pragma unroll
        for (int c = 0; c < G / 8; ++c) {
            const uint4 w = *reinterpret_cast<const uint4 *>(row + c * 16);
            const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[8 * c + 2 * i] = __uint_as_float(ws[i] << 16);
                x[8 * c + 2 * i + 1] = __uint_as_float(ws[i] & 0xffff0000u);
            }
        }
    } else {
#pragma unroll
        for (int c = 0; c < G / 4; ++c) {
            const float4 w = *reinterpret_cast<const float4 *>(row + c * 16);
            x[4 * c] = w.x; x[4 * c + 1] = w.y; x[4 * c + 2] = w.z; x[4 * c + 3] = w.w;
        }
    }
}

// Adjacent-pair binary tree over N = 2^m values held in registers: the level-by-level pairing
// z'[k] = z[2k] + z[2k+1] is the same expression tree as "left half + right half", recursively.
template <int N>
__device__ __forceinline__ float tree_sum(const float *z)
{
    if constexpr (N == 1) return z[0];
    else return tree_sum<N / 2>(z) + tree_sum<N / 2>(z + N / 2);
}

// Unnormalised Sylvester butterfly on a whole tile in registers, stages h = 1, 2, ..., G/2.
template <int G>
__device__ __forceinline__ void butterfly(float *x)
{
#pragma unroll
    for (int h = 1; h < G; h <<= 1) {
#pragma unroll
        for (int i = 0; i < G; ++i) {
            if ((i & h) == 0) {
                const float p = x[i], q = x[i + h];
                x[i] = p + q;
                x[i + h] = p - q;
            }
        }
    }
}

// -------------------------------------------------------------- K0: entropy

template <int G, bool BF16>
__global__ __launch_bounds__((Batch<G, BF16 ? 2 : 4>::TILES))
void k_entropy(const void *__restrict__ in, float *__restrict__ H, uint32_t T, float eps_l1, float eps_log)
{
    using B = Batch<G, BF16 ? 2 : 4>;
    __shared__ __attribute__((aligned(16))) uint8_t lds[B::LDS_BYTES];
    const uint64_t j0 = (uint64_t)blockIdx.x * B::TILES;
    const uint32_t left = (uint32_t)(T - j0);
    const uint32_t nvalid = left < (uint32_t)B::TILES ? left : (uint32_t)B::TILES;
    stage_in<G, BF16 ? 2 : 4>(in, j0, nvalid, lds);
    __syncthreads();
    if (threadIdx.x >= nvalid) return;

    float a[G];
    read_tile<G, BF16>(lds + threadIdx.x * B::STRIDE, a);
#pragma unroll
    for (int k = 0; k < G; ++k) a[k] = __builtin_fabsf(a[k]);
    const float L1 = tree_sum<G>(a);
    const float invL = 1.0f / (L1 + eps_l1);
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const float p = a[k] * invL;
        const float u = p + eps_log;
        a[k] = p * log_contract(u);
    }
    H[j0 + threadIdx.x] = 0.0f - tree_sum<G>(a);
}

// ------------------------------------ K3: transform + quantize + pack

// Payload unit: a tile's payload is b units of G/8 bytes (b = 3 or 4).
template <int G> struct Unit;
template <> struct Unit<32>  { using type = uint32_t; };
template <> struct Unit<64>  { using type = uint2; };
template <> struct Unit<128> { using type = uint4; };

// Median of three unsigned integers in one vector instruction.
__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Eq. 3 on my tile, read from its LDS row: magnitude of the largest and second-largest element
// (with multiplicity) and the lowest index of the largest.
template <int G, bool BF16>
__device__ __forceinline__ void top2(const uint8_t *row, float *a1_out, float *a2_out, uint32_t *d_out)
{
    if constexpr (BF16) {
        // A bf16 magnitude has 16 free low bits: key = |bits| << 16 | (G-1-k) orders by magnitude, then by
        // lower index, under unsigned integer max.  Even and odd elements run in separate chains (the
        // even chain keeps its keys shifted left by one, which drops the sign bit for free).
        uint32_t e1 = 0, e2 = 0, o1 = 0, o2 = 0;
#pragma unroll
        for (int c = 0; c < G / 8; ++c) {
            const uint4 w = *reinterpret_cast<const uint4 *>(row + c * 16);
            const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t k_even = 8 * c + 2 * i, k_odd = k_even + 1;
                const uint32_t ke = (ws[i] << 17) | ((G - 1 - k_even) << 1);
                const uint32_t ko = (ws[i] & 0x7fff0000u) | (G - 1 - k_odd);
                e2 = umed3(e1, e2, ke);   // second largest of {e1 >= e2, ke}
                e1 = e1 > ke ? e1 : ke;
                o2 = umed3(o1, o2, ko);
                o1 = o1 > ko ? o1 : ko;
            }
        }
        e1 >>= 1; e2 >>= 1;
        const uint32_t k1 = e1 > o1 ? e1 : o1;
        const uint32_t lo = e1 > o1 ? o1 : e1;
        const uint32_t hi2 = e2 > o2 ? e2 : o2;
        const uint32_t k2 = lo > hi2 ? lo : hi2;
        *a1_out = __uint_as_float(k1 & 0x7fff0000u);
        *a2_out = __uint_as_float(k2 & 0x7fff0000u);
        *d_out = (G - 1) - (k1 & 0x7fu);
    } else {
        float a1 = -1.0f, a2 = 0.0f;     // magnitudes are >= 0: the first element always replaces a1
        uint32_t d = 0;
#pragma unroll
        for (int c = 0; c < G / 4; ++c) {
            const float4 w = *reinterpret_cast<const float4 *>(row + c * 16);
            const float ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float a = __builtin_fabsf(ws[i]);
                const bool gt = a > a1;
                a2 = gt ? a1 : __builtin_fmaxf(a2, a);
                d = gt ? (uint32_t)(4 * c + i) : d;
                a1 = gt ? a : a1;
            }
        }
        *a1_out = a1;
        *a2_out = __builtin_fmaxf(a2, 0.0f);
        *d_out = d;
    }
}

template <int G, bool BF16>
__global__ __launch_bounds__((Batch<G, BF16 ? 2 : 4>::TILES))
void k_quant_pack(const void *__restrict__ in, uint8_t *__restrict__ packed, Layout lay, uint32_t T, float tau,
                  float eps_ratio)
{
    constexpr int ES = BF16 ? 2 : 4;
    using B = Batch<G, ES>;
    using U = typename Unit<G>::type;
    __shared__ __attribute__((aligned(16))) uint8_t lds[B::LDS_BYTES];
    __shared__ __attribute__((aligned(16))) U pay[B::TILES * 4];
    const int tid = threadIdx.x;
    const uint64_t j0 = (uint64_t)blockIdx.x * B::TILES;
    const uint32_t left = (uint32_t)(T - j0);
    const uint32_t nvalid = left < (uint32_t)B::TILES ? left : (uint32_t)B::TILES;
    stage_in<G, ES>(in, j0, nvalid, lds);

    // width and payload position of my tile: bit map word and rank-table entry of my 64-tile group
    const uint64_t j = j0 + tid;
    const bool valid = (uint32_t)tid < nvalid;
    const uint64_t *bitmap = reinterpret_cast<const uint64_t *>(packed + lay.bitmap);
    const uint32_t *ranks = reinterpret_cast<const uint32_t *>(packed + lay.ranks);
    const uint32_t rank0 = ranks[j0 >> 6];
    uint32_t b = 3, rel = 0;          // rel: my payload position inside the batch, in units
    uint32_t total4 = 0;              // 4-bit tiles in the batch
#pragma unroll
    for (int w = 0; w < (B::TILES + 63) / 64; ++w) {
        const uint64_t jw = (j0 >> 6) + w;
        const uint64_t word = jw * 64 < T ? bitmap[jw] : 0ull;
        if (w == (tid >> 6)) {
            const uint32_t bit = (uint32_t)tid & 63u;
            b = 3u + (uint32_t)((word >> bit) & 1ull);
            rel = 3u * (uint32_t)tid + total4 + (uint32_t)__popcll(word & ((1ull << bit) - 1ull));
        }
        total4 += (uint32_t)__popcll(word);
    }
    __syncthreads();

    if (valid) {
        uint8_t *row = lds + tid * B::STRIDE;
        float a1, a2;
        uint32_t d;
        top2<G, BF16>(row, &a1, &a2, &d);
        const bool flag = a1 > tau * (a2 + eps_ratio);
        if (flag && d != 0) {
            // P_d: swap elements 0 and d inside my LDS row
            if constexpr (BF16) {
                uint16_t *r16 = reinterpret_cast<uint16_t *>(row);
                const uint16_t v0 = r16[0], vd = r16[d];
                r16[0] = vd; r16[d] = v0;
            } else {
                float *r32 = reinterpret_cast<float *>(row);
                const float v0 = r32[0], vd = r32[d];
                r32[0] = vd; r32[d] = v0;
            }
        }
        float x[G];
        read_tile<G, BF16>(row, x);
        if (flag) {
            butterfly<G>(x);
#pragma unroll
            for (int k = 0; k < G; ++k) x[k] = x[k] * TileConst<G>::c;
        }
        float mn = x[0], mx = x[0];
#pragma unroll
        for (int k = 1; k < G; ++k) { mn = __builtin_fminf(mn, x[k]); mx = __builtin_fmaxf(mx, x[k]); }
        mn = mn + 0.0f;
        mx = mx + 0.0f;

        // asymmetric quantizer, binary16 metadata rounded outwards
        const float Lv = (b == 4u) ? 15.0f : 7.0f;
        const uint32_t z16 = f16_down(mn);
        const float mnf = f16_widen(z16);
        const float s = (mx - mnf) / Lv;
        uint32_t s16 = f16_up(s);
        if ((s16 & 0x7fffu) == 0) s16 = 0x3c00u;
        const float sf = f16_widen(s16);
        const float rcp = 1.0f / sf;

        // codes, four at a time: q0 + m q1 + m^2 q2 + m^3 q3 is an exact integer below 2^16 in fp32
        const float m1 = (b == 4u) ? 16.0f : 8.0f;
        const float m2 = m1 * m1, m3 = m2 * m1;
        uint32_t v[G / 4];
#pragma unroll
        for (int g = 0; g < G / 4; ++g) {
            float q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                q[i] = __builtin_fminf(__builtin_fmaxf(__builtin_rintf((x[4 * g + i] - mnf) * rcp), 0.0f), Lv);
            const float acc = __builtin_fmaf(q[3], m3, __builtin_fmaf(q[2], m2, __builtin_fmaf(q[1], m1, q[0])));
            v[g] = (uint32_t)acc;
        }
        // LSB-first bit string of the tile as dwords
        uint32_t dw[G / 8];
        if (b == 4u) {
#pragma unroll
            for (int i = 0; i < G / 8; ++i) dw[i] = v[2 * i] | (v[2 * i + 1] << 16);
        } else {
            // 12-bit groups: eight of them fill three dwords
#pragma unroll
            for (int i = 0; i < G / 32; ++i) {
                const uint32_t *p = v + 8 * i;
                dw[3 * i + 0] = p[0] | (p[1] << 12) | (p[2] << 24);
                dw[3 * i + 1] = (p[2] >> 8) | (p[3] << 4) | (p[4] << 16) | (p[5] << 28);
                dw[3 * i + 2] = (p[5] >> 4) | (p[6] << 8) | (p[7] << 20);
            }
#pragma unroll
            for (int i = 3 * (G / 32); i < G / 8; ++i) dw[i] = 0;
        }
        U *dst = pay + rel;
        constexpr int DPU = G / 32;     // dwords per unit
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u < 3 || b == 4u) {
                if constexpr (G == 32) dst[u] = dw[u];
                else if constexpr (G == 64) dst[u] = make_uint2(dw[2 * u], dw[2 * u + 1]);
                else dst[u] = make_uint4(dw[4 * u], dw[4 * u + 1], dw[4 * u + 2], dw[4 * u + 3]);
            }
        }
        (void)DPU;
        reinterpret_cast<uint16_t *>(packed + lay.scale)[j] = (uint16_t)s16;
        reinterpret_cast<uint16_t *>(packed + lay.zero)[j] = (uint16_t)z16;
        packed[lay.pivot + j] = flag ? (uint8_t)(0x80u | d) : (uint8_t)0;
    }
    __syncthreads();

    // the batch's payload is one contiguous span: copy it out dword by dword, coalesced
    const uint32_t span_dw = (G / 32) * (3u * nvalid + total4);
    uint32_t *gdst = reinterpret_cast<uint32_t *>(packed + lay.payload) + (uint64_t)(G / 32) * (3ull * j0 + rank0);
    const uint32_t *psrc = reinterpret_cast<const uint32_t *>(pay);
    for (uint32_t i = tid; i < span_dw; i += B::TILES) gdst[i] = psrc[i];
}

// ------------------------------------------------------------- K4: decode

template <int G, bool OUT_BF16>
__global__ __launch_bounds__((Batch<G, OUT_BF16 ? 2 : 4>::TILES))
void k_decode(const uint8_t *__restrict__ packed, void *__restrict__ out, Layout lay, uint32_t T)
{
    constexpr int ES = OUT_BF16 ? 2 : 4;
    using B = Batch<G, ES>;
    using U = typename Unit<G>::type;
    __shared__ __attribute__((aligned(16))) uint8_t lds[B::LDS_BYTES];
    __shared__ __attribute__((aligned(16))) U pay[B::TILES * 4];
    const int tid = threadIdx.x;
    const uint64_t j0 = (uint64_t)blockIdx.x * B::TILES;
    const uint32_t left = (uint32_t)(T - j0);
    const uint32_t nvalid = left < (uint32_t)B::TILES ? left : (uint32_t)B::TILES;
    const uint64_t j = j0 + tid;
    const bool valid = (uint32_t)tid < nvalid;

    const uint64_t *bitmap = reinterpret_cast<const uint64_t *>(packed + lay.bitmap);
    const uint32_t *ranks = reinterpret_cast<const uint32_t *>(packed + lay.ranks);
    const uint32_t rank0 = ranks[j0 >> 6];
    uint32_t b = 3, rel = 0, total4 = 0;
#pragma unroll
    for (int w = 0; w < (B::TILES + 63) / 64; ++w) {
        const uint64_t jw = (j0 >> 6) + w;
        const uint64_t word = jw * 64 < T ? bitmap[jw] : 0ull;
        if (w == (tid >> 6)) {
            const uint32_t bit = (uint32_t)tid & 63u;
            b = 3u + (uint32_t)((word >> bit) & 1ull);
            rel = 3u * (uint32_t)tid + total4 + (uint32_t)__popcll(word & ((1ull << bit) - 1ull));
        }
        total4 += (uint32_t)__popcll(word);
    }

    // stage the batch's payload span
    const uint32_t span_dw = (G / 32) * (3u * nvalid + total4);
    const uint32_t *gsrc = reinterpret_cast<const uint32_t *>(packed + lay.payload) + (uint64_t)(G / 32) * (3ull * j0 + rank0);
    uint32_t *pdst = reinterpret_cast<uint32_t *>(pay);
    for (uint32_t i = tid; i < span_dw; i += B::TILES) pdst[i] = gsrc[i];

    uint32_t s16 = 0, z16 = 0, pv = 0;
    if (valid) {
        s16 = reinterpret_cast<const uint16_t *>(packed + lay.scale)[j];
        z16 = reinterpret_cast<const uint16_t *>(packed + lay.zero)[j];
        pv = packed[lay.pivot + j];
    }
    __syncthreads();

    uint8_t *row = lds + tid * B::STRIDE;
    if (valid) {
        const float sf = f16_widen(s16), mnf = f16_widen(z16);
        // my 3 or 4 units (the 4th is read in any case: it stays inside the array)
        uint32_t dw[G / 8];
        const U *src = pay + rel;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const U t = src[u];
            if constexpr (G == 32) dw[u] = t;
            else if constexpr (G == 64) { dw[2 * u] = t.x; dw[2 * u + 1] = t.y; }
            else { dw[4 * u] = t.x; dw[4 * u + 1] = t.y; dw[4 * u + 2] = t.z; dw[4 * u + 3] = t.w; }
        }
        // bring three-bit codes onto nibble boundaries: 24 bits (8 codes) -> 32 bits
        uint32_t nib[G / 8];
        if (b == 4u) {
#pragma unroll
            for (int i = 0; i < G / 8; ++i) nib[i] = dw[i];
        } else {
#pragma unroll
            for (int i = 0; i < G / 8; ++i) {
                // codes 8i .. 8i+7 occupy bits [24i, 24i+24) of the string
                const int lo = (24 * i) >> 5, sh = (24 * i) & 31;
                uint32_t t = dw[lo] >> sh;
                if (sh > 8) t |= dw[lo + 1] << (32 - sh);
                t &= 0x00ffffffu;
                t = (t & 0x00000fffu) | ((t & 0x00fff000u) << 4);
                t = (t & 0x003f003fu) | ((t & 0x0fc00fc0u) << 2);
                t = (t & 0x07070707u) | ((t & 0x38383838u) << 1);
                nib[i] = t;
            }
        }
        // de-quantize: even codes sit in the low nibbles of the bytes, odd codes in the high nibbles
        // (scaled by 16, undone exactly by a scale of sf/16)
        const float sf16 = sf * 0.0625f;
        float x[G];
#pragma unroll
        for (int i = 0; i < G / 8; ++i) {
            const uint32_t lo = nib[i] & 0x0f0f0f0fu, hi = nib[i] & 0xf0f0f0f0u;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                x[8 * i + 2 * c] = __builtin_fmaf((float)((lo >> (8 * c)) & 0xffu), sf, mnf);
                x[8 * i + 2 * c + 1] = __builtin_fmaf((float)((hi >> (8 * c)) & 0xffu), sf16, mnf);
            }
        }
        if (pv & 0x80u) {
            butterfly<G>(x);
#pragma unroll
            for (int k = 0; k < G; ++k) x[k] = x[k] * TileConst<G>::c;
        }
        // my tile into its LDS row, narrowed to the output type
        if constexpr (OUT_BF16) {
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            typedef float floatx2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int c = 0; c < G / 8; ++c) {
                uint32_t ws[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const floatx2 pr = {x[8 * c + 2 * i], x[8 * c + 2 * i + 1]};
                    ws[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
                }
                *reinterpret_cast<uint4 *>(row + c * 16) = make_uint4(ws[0], ws[1], ws[2], ws[3]);
            }
        } else {
#pragma unroll
            for (int c = 0; c < G / 4; ++c)
                *reinterpret_cast<float4 *>(row + c * 16) = make_float4(x[4 * c], x[4 * c + 1], x[4 * c + 2], x[4 * c + 3]);
        }
        const uint32_t d = pv & 0x7fu;
        if ((pv & 0x80u) && d != 0) {
            // undo P_d inside my row
            if constexpr (OUT_BF16) {
                uint16_t *r16 = reinterpret_cast<uint16_t *>(row);
                const uint16_t v0 = r16[0], vd = r16[d];
                r16[0] = vd; r16[d] = v0;
            } else {
                float *r32 = reinterpret_cast<float *>(row);
                const float v0 = r32[0], vd = r32[d];
                r32[0] = vd; r32[d] = v0;
            }
        }
    }
    __syncthreads();
    stage_out<G, ES>(out, j0, nvalid, lds);
}

}  // namespace tahq
