// Streaming kernels: entropy (Eq. 1-2), transform + quantize + pack (Eq. 3-4, Sec. 3.4),
// decode (Alg. 1 step 5).
#pragma once
#include "tahq_common.hpp"

namespace tahq {

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

}  // namespace tahq
