// Backward-pass compressor: b-bit fixed-point codes of c*g and back (Sec. 3.5 / Alg. 1 steps 6-7 and
// the appendix's gradient scaling g_hat = Q(c g)/c).
//
// Mapping: ONE LANE OWNS ONE CHUNK of 32 consecutive elements, whose codes fill exactly BITS 32-bit
// words.  A workgroup stages 256 chunks through LDS with coalesced 128-bit global accesses on both
// sides, like the forward codec's kernels; the work per element is a handful of vector instructions, so
// these kernels are bound by HBM.
#pragma once
#include "tahq_stream_kernels.hpp"

namespace tahq {

constexpr int kNaiveChunk = 32;      // elements per lane
constexpr int kNaiveChunks = 256;    // chunks (lanes) per workgroup

struct NaiveHeader { uint32_t w[16]; };

// Payload words of a workgroup sit in LDS at a skewed index, so that both the lane-per-chunk accesses
// (stride BITS words) and the coalesced copies (stride 1) spread over the banks.
__device__ __forceinline__ uint32_t skew(uint32_t p) { return p + (p >> 5); }

template <int BITS, bool BF16>
__global__ __launch_bounds__(kNaiveChunks)
void k_naive_encode(const void *__restrict__ in, uint8_t *__restrict__ packed, NaiveHeader hdr, uint32_t nchunks,
                    float scale)
{
    constexpr int ES = BF16 ? 2 : 4;
    using B = Batch<kNaiveChunk, ES>;
    static_assert(B::TILES == kNaiveChunks, "one lane per chunk");
    __shared__ __attribute__((aligned(16))) uint8_t rows[B::LDS_BYTES];
    __shared__ uint32_t pay[kNaiveChunks * BITS + kNaiveChunks * BITS / 32 + 1];
    const int tid = threadIdx.x;
    const uint32_t j0 = blockIdx.x * kNaiveChunks;
    const uint32_t left = nchunks - j0;
    const uint32_t nvalid = left < (uint32_t)kNaiveChunks ? left : (uint32_t)kNaiveChunks;
    if (blockIdx.x == 0 && tid < 16) reinterpret_cast<uint32_t *>(packed)[tid] = hdr.w[tid];

    uint4 v[B::CHUNKS];
    if (nvalid == (uint32_t)kNaiveChunks) {
        load_batch<kNaiveChunk, ES, true, true>(in, j0, nvalid, v);
        store_batch<kNaiveChunk, ES, true>(v, nvalid, rows);
    } else {
        load_batch<kNaiveChunk, ES, false>(in, j0, nvalid, v);
        store_batch<kNaiveChunk, ES, false>(v, nvalid, rows);
    }
    __syncthreads();
    if ((uint32_t)tid < nvalid) {
        float x[kNaiveChunk];
        read_tile<kNaiveChunk, BF16>(rows + tid * B::STRIDE, x);
        constexpr float lo = -(float)(1u << (BITS - 1));
        constexpr float hi = (float)((1u << (BITS - 1)) - 1u);
        constexpr uint32_t mask = (1u << BITS) - 1u;
        uint64_t acc = 0;
        int have = 0, word = 0;
#pragma unroll
        for (int i = 0; i < kNaiveChunk; ++i) {
            const float y = scale * x[i];
            float r = __builtin_rintf(y);
            r = __builtin_fmaxf(r, lo);
            r = __builtin_fminf(r, hi);
            const uint32_t field = (uint32_t)(int32_t)r & mask;
            acc |= (uint64_t)field << have;
            have += BITS;
            if (have >= 32) {
                pay[skew((uint32_t)tid * BITS + word)] = (uint32_t)acc;
                acc >>= 32;
                have -= 32;
                ++word;
            }
        }
    }
    __syncthreads();
    // coalesced copy of the workgroup's nvalid*BITS payload words
    uint32_t *dst = reinterpret_cast<uint32_t *>(packed + 64) + (uint64_t)j0 * BITS;
    const uint32_t nwords = nvalid * BITS;
#pragma unroll
    for (int i = 0; i < BITS; ++i) {
        const uint32_t p = (uint32_t)i * kNaiveChunks + tid;
        if (p < nwords) __builtin_nontemporal_store(pay[skew(p)], dst + p);
    }
}

template <int BITS, bool OUT_BF16>
__global__ __launch_bounds__(kNaiveChunks)
void k_naive_decode(const uint8_t *__restrict__ packed, void *__restrict__ out, uint32_t nchunks, float inv_scale)
{
    constexpr int ES = OUT_BF16 ? 2 : 4;
    using B = Batch<kNaiveChunk, ES>;
    __shared__ __attribute__((aligned(16))) uint8_t rows[B::LDS_BYTES];
    __shared__ uint32_t pay[kNaiveChunks * BITS + kNaiveChunks * BITS / 32 + 1];
    const int tid = threadIdx.x;
    const uint32_t j0 = blockIdx.x * kNaiveChunks;
    const uint32_t left = nchunks - j0;
    const uint32_t nvalid = left < (uint32_t)kNaiveChunks ? left : (uint32_t)kNaiveChunks;
    const uint32_t *src = reinterpret_cast<const uint32_t *>(packed + 64) + (uint64_t)j0 * BITS;
    const uint32_t nwords = nvalid * BITS;
    // (from a clamped index: a load behind a bounds-check branch would wait for the one before it; words past the
    // end of a ragged workgroup are never used)
    uint32_t got[BITS];
#pragma unroll
    for (int i = 0; i < BITS; ++i) {
        const uint32_t p = (uint32_t)i * kNaiveChunks + tid;
        got[i] = __builtin_nontemporal_load(src + (p < nwords ? p : nwords - 1));
    }
#pragma unroll
    for (int i = 0; i < BITS; ++i) pay[skew((uint32_t)i * kNaiveChunks + tid)] = got[i];
    __syncthreads();
    if ((uint32_t)tid < nvalid) {
        uint32_t w[BITS];
#pragma unroll
        for (int i = 0; i < BITS; ++i) w[i] = pay[skew((uint32_t)tid * BITS + i)];
        float x[kNaiveChunk];
#pragma unroll
        for (int i = 0; i < kNaiveChunk; ++i) {
            const int bit = i * BITS, idx = bit >> 5, sh = bit & 31;
            int32_t q;
            if (sh + BITS <= 32) {
                // the field lies inside one word: move it to the top, shift back down with the sign
                q = (int32_t)(w[idx] << (32 - BITS - sh)) >> (32 - BITS);
            } else {
                const uint32_t window = (w[idx] >> sh) | (w[idx + 1] << (32 - sh));
                q = (int32_t)(window << (32 - BITS)) >> (32 - BITS);
            }
            x[i] = (float)q * inv_scale;
        }
        uint8_t *row = rows + tid * B::STRIDE;
        if constexpr (OUT_BF16) {
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            typedef float floatx2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int c = 0; c < kNaiveChunk / 8; ++c) {
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
            for (int c = 0; c < kNaiveChunk / 4; ++c)
                *reinterpret_cast<float4 *>(row + c * 16) = make_float4(x[4 * c], x[4 * c + 1], x[4 * c + 2], x[4 * c + 3]);
        }
    }
    __syncthreads();
    if (nvalid == (uint32_t)kNaiveChunks) stage_out<kNaiveChunk, ES, true>(out, j0, nvalid, rows);
    else stage_out<kNaiveChunk, ES, false>(out, j0, nvalid, rows);
}

}  // namespace tahq
