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

// A batch's tiles travel global -> registers -> padded LDS rows, in two steps, so that the loads of the
// next batch can be in flight while the current one is being processed.  Thread t moves the 16-byte
// chunks t, t + TILES, t + 2 TILES, ... of the batch (coalesced).  FULL: all TILES tiles exist, no
// per-thread conditions (so that the compiler can count outstanding memory operations exactly).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16-byte global load; STREAM marks data that will not be read again soon (non-temporal hint).
template <bool STREAM>
__device__ __forceinline__ uint4 load16(const uint8_t *p)
{
    if constexpr (STREAM) {
        const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
        return make_uint4(t.x, t.y, t.z, t.w);
    } else {
        return *reinterpret_cast<const uint4 *>(p);
    }
}

template <int G, int ESIZE, bool FULL, bool STREAM = false>
__device__ __forceinline__ void load_batch(const void *__restrict__ in, uint64_t j0, uint32_t nvalid,
                                           uint4 (&v)[Batch<G, ESIZE>::CHUNKS], int tid = (int)threadIdx.x)
{
    using B = Batch<G, ESIZE>;
    const uint8_t *src = static_cast<const uint8_t *>(in) + j0 * B::BYTES;
#pragma unroll
    for (int i = 0; i < B::CHUNKS; ++i) {
        const uint32_t q = (uint32_t)i * B::TILES + tid;
        if constexpr (FULL) {
            v[i] = load16<STREAM>(src + (uint64_t)q * 16);
        } else {
            v[i] = make_uint4(0u, 0u, 0u, 0u);
            if (q / B::CHUNKS < nvalid) v[i] = load16<STREAM>(src + (uint64_t)q * 16);
        }
    }
}

template <int G, int ESIZE, bool FULL>
__device__ __forceinline__ void store_batch(const uint4 (&v)[Batch<G, ESIZE>::CHUNKS], uint32_t nvalid, uint8_t *lds,
                                            int tid = (int)threadIdx.x)
{
    using B = Batch<G, ESIZE>;
#pragma unroll
    for (int i = 0; i < B::CHUNKS; ++i) {
        const uint32_t q = (uint32_t)i * B::TILES + tid;
        const uint32_t tile = q / B::CHUNKS, sub = q % B::CHUNKS;
        if (FULL || tile < nvalid) *reinterpret_cast<uint4 *>(lds + tile * B::STRIDE + sub * 16) = v[i];
    }
}

// Coalesced copy of `nvalid` tiles from padded LDS rows to global memory.
template <int G, int ESIZE, bool FULL>
__device__ __forceinline__ void stage_out(void *__restrict__ out, uint64_t j0, uint32_t nvalid, const uint8_t *lds)
{
    using B = Batch<G, ESIZE>;
    uint8_t *dst = static_cast<uint8_t *>(out) + j0 * B::BYTES;
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < B::CHUNKS; ++i) {
        const uint32_t q = (uint32_t)i * B::TILES + tid;
        const uint32_t tile = q / B::CHUNKS, sub = q % B::CHUNKS;
        if (FULL || tile < nvalid) {
            // streaming store: the decoded tensor is not read again by this library
            const uint4 val = *reinterpret_cast<const uint4 *>(lds + tile * B::STRIDE + sub * 16);
            const u32x4 vv = {val.x, val.y, val.z, val.w};
            __builtin_nontemporal_store(vv, reinterpret_cast<u32x4 *>(dst + (uint64_t)q * 16));
        }
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

// Eq. 1-2 for my tile, read from its LDS row.
template <int G, bool BF16>
__device__ __forceinline__ float entropy_of_row(const uint8_t *row, float eps_l1, float eps_log)
{
    float a[G];
    read_tile<G, BF16>(row, a);
#pragma unroll
    for (int k = 0; k < G; ++k) a[k] = __builtin_fabsf(a[k]);
    const float L1 = tree_sum<G>(a);
    const float invL = 1.0f / (L1 + eps_l1);
#pragma unroll
    for (int k = 0; k < G; ++k) a[k] = a[k] * log_contract(__builtin_fmaf(a[k], invL, eps_log));
    return 0.0f - invL * tree_sum<G>(a);
}

constexpr int kDigit0Bits = 10;                  // first radix digit of the selection: key bits 31..22
static_assert((1u << kDigit0Bits) == kDigit0Bins, "digit 0 width");

// Persistent workgroups: workgroup w handles a contiguous run of full batches.  The next batch's loads
// are issued before the current batch is processed, and a batch's result is stored one iteration later,
// just before those loads, so that no wait for loads ever has a younger store in front of it.
// The ragged last batch (T not a multiple of TILES) is handled after the loop by one workgroup.
//
// If `hist0` is given, the kernel also builds the first histogram of the selection (Sec. 3.2, top-p%): per
// ranking unit of `unit_batches` batches, counts of the keys' top 10 bits (bin_scale == 0) or of the entropies'
// linear bins (bin_scale > 0), `hist_stride` bins per unit, accumulated in LDS and flushed with global atomics
// when the workgroup moves to another unit and at its end.  This needs units that are whole numbers of batches
// (the caller checks; otherwise it passes no histogram).
template <int G, bool BF16>
__global__ __launch_bounds__((Batch<G, BF16 ? 2 : 4>::TILES))
void k_entropy(const void *__restrict__ in, float *__restrict__ H, uint32_t T, float eps_l1, float eps_log,
               uint32_t *__restrict__ hist0, uint32_t unit_batches, uint32_t hist_stride, float bin_scale)
{
    constexpr int ES = BF16 ? 2 : 4;
    using B = Batch<G, ES>;
    __shared__ __attribute__((aligned(16))) uint8_t lds[B::LDS_BYTES];
    static_assert(kLinBins >= kDigit0Bins, "one LDS histogram serves both kinds of bins");
    __shared__ uint32_t lh[kLinBins];
    const int tid = threadIdx.x;
    const uint32_t nfull = T / B::TILES, tail = T % B::TILES;
    const uint8_t *row = lds + tid * B::STRIDE;
    const uint32_t per = (nfull + gridDim.x - 1) / gridDim.x;
    const uint32_t first = blockIdx.x * per;
    const uint32_t last = first + per < nfull ? first + per : nfull;      // my batches: [first, last)

    if (hist0) {
        for (int i = tid; i < (int)hist_stride; i += B::TILES) lh[i] = 0;
    }
    auto flush = [&](uint32_t unit) {
        __syncthreads();
        for (int i = tid; i < (int)hist_stride; i += B::TILES) {
            const uint32_t c = lh[i];
            if (c) { atomicAdd(&hist0[(uint64_t)unit * hist_stride + i], c); lh[i] = 0; }
        }
        __syncthreads();
    };

    uint4 v[B::CHUNKS];
    // non-temporal loads: the tensor is much larger than any cache, and keeping part of it for the second
    // pass measured slower than streaming all of it
    auto load_full = [&](uint32_t batch) {
        load_batch<G, ES, true, true>(in, (uint64_t)batch * B::TILES, B::TILES, v);
    };
    if (first < last) load_full(first);
    float h_prev = 0.0f;
    uint64_t j_prev = 0;
    bool have_prev = false;
    uint32_t cur_unit = hist0 && first < last ? first / unit_batches : 0u;
    for (uint32_t batch = first; batch < last; ++batch) {
        if (hist0) {
            const uint32_t unit = batch / unit_batches;
            if (unit != cur_unit) { flush(cur_unit); cur_unit = unit; }
        }
        store_batch<G, ES, true>(v, B::TILES, lds);
        __syncthreads();
        if (have_prev) H[j_prev] = h_prev;
        if (batch + 1 < last) load_full(batch + 1);
        h_prev = entropy_of_row<G, BF16>(row, eps_l1, eps_log);
        if (hist0)
            atomicAdd(&lh[bin_scale > 0.0f ? linear_bin(h_prev, bin_scale) : order_key(h_prev) >> (32 - kDigit0Bits)], 1u);
        j_prev = (uint64_t)batch * B::TILES + tid;
        have_prev = true;
        __syncthreads();
    }
    if (have_prev) H[j_prev] = h_prev;
    if (hist0 && first < last) flush(cur_unit);

    if (tail != 0 && blockIdx.x == gridDim.x - 1) {
        // never combined with a histogram: a ragged batch means units are not whole batches
        const uint64_t j0 = (uint64_t)nfull * B::TILES;
        load_batch<G, ES, false>(in, j0, tail, v);
        store_batch<G, ES, false>(v, tail, lds);
        __syncthreads();
        if ((uint32_t)tid < tail) H[j0 + tid] = entropy_of_row<G, BF16>(row, eps_l1, eps_log);
    }
}

// ---------------------- entropy of allocation tiles wider than a quantization tile

// Sec. 3.2 with A = m*G, m > 1: Eq. 1's norm and Eq. 2's sum run over the A channels of an allocation
// tile.  Both are accumulated per quantization tile by the pairwise tree and then across the m tiles
// from left to right.  In general the work splits into two streaming passes with a small reduction after
// each:
//   WEIGHTED = false: part[j] = sum over tile j of |v|
//   WEIGHTED = true:  part[j] = sum over tile j of |v| log(|v| * r + varsigma), r = inv_norm[j / m] (the common factor r
//                     of Eq. 2's sum is applied once, by the reduction)
// One workgroup per batch of tiles, one lane per tile.
template <int G, bool BF16, bool WEIGHTED>
__global__ __launch_bounds__((Batch<G, BF16 ? 2 : 4>::TILES))
void k_tile_partial(const void *__restrict__ in, const float *__restrict__ inv_norm, float *__restrict__ part,
                    uint32_t T, uint32_t m, float eps_log)
{
    constexpr int ES = BF16 ? 2 : 4;
    using B = Batch<G, ES>;
    __shared__ __attribute__((aligned(16))) uint8_t lds[B::LDS_BYTES];
    const int tid = threadIdx.x;
    const uint64_t j0 = (uint64_t)blockIdx.x * B::TILES;
    const uint32_t left = T - (uint32_t)j0;
    const uint32_t nvalid = left < (uint32_t)B::TILES ? left : (uint32_t)B::TILES;
    uint4 v[B::CHUNKS];
    if (nvalid == (uint32_t)B::TILES) {
        load_batch<G, ES, true, true>(in, j0, nvalid, v);
        store_batch<G, ES, true>(v, nvalid, lds);
    } else {
        load_batch<G, ES, false>(in, j0, nvalid, v);
        store_batch<G, ES, false>(v, nvalid, lds);
    }
    __syncthreads();
    if ((uint32_t)tid >= nvalid) return;
    const uint32_t j = (uint32_t)j0 + tid;
    float a[G];
    read_tile<G, BF16>(lds + tid * B::STRIDE, a);
#pragma unroll
    for (int k = 0; k < G; ++k) a[k] = __builtin_fabsf(a[k]);
    if constexpr (WEIGHTED) {
        const float invL = inv_norm[j / m];
#pragma unroll
        for (int k = 0; k < G; ++k) a[k] = a[k] * log_contract(__builtin_fmaf(a[k], invL, eps_log));
    }
    part[j] = tree_sum<G>(a);
}

// The same result in ONE pass over the tensor when a workgroup's batch holds whole allocation tiles
// (m divides TILES): the per-tile sums meet in LDS, the first lane of every allocation tile adds its m
// values from left to right, and the tile's magnitudes wait in registers meanwhile.
template <int G, bool BF16>
__global__ __launch_bounds__((Batch<G, BF16 ? 2 : 4>::TILES), (G * (BF16 ? 2 : 4) <= 128 ? 4 : 1))
void k_alloc_entropy(const void *__restrict__ in, float *__restrict__ H, uint32_t T, uint32_t m, float eps_l1,
                     float eps_log)
{
    constexpr int ES = BF16 ? 2 : 4;
    using B = Batch<G, ES>;
    __shared__ __attribute__((aligned(16))) uint8_t lds[B::LDS_BYTES];
    __shared__ float part[B::TILES];
    __shared__ float inv_norm[B::TILES];
    const int tid = threadIdx.x;
    const uint64_t j0 = (uint64_t)blockIdx.x * B::TILES;
    const uint32_t left = T - (uint32_t)j0;
    const uint32_t nvalid = left < (uint32_t)B::TILES ? left : (uint32_t)B::TILES;   // a multiple of m
    uint4 v[B::CHUNKS];
    if (nvalid == (uint32_t)B::TILES) {
        load_batch<G, ES, true, true>(in, j0, nvalid, v);
        store_batch<G, ES, true>(v, nvalid, lds);
    } else {
        load_batch<G, ES, false>(in, j0, nvalid, v);
        store_batch<G, ES, false>(v, nvalid, lds);
    }
    __syncthreads();
    const bool valid = (uint32_t)tid < nvalid;
    const bool first = valid && (uint32_t)tid % m == 0;      // first quantization tile of its allocation tile
    float a[G];
    if (valid) {
        read_tile<G, BF16>(lds + tid * B::STRIDE, a);
#pragma unroll
        for (int k = 0; k < G; ++k) a[k] = __builtin_fabsf(a[k]);
        part[tid] = tree_sum<G>(a);
    }
    __syncthreads();
    if (first) {
        float acc = 0.0f;
        for (uint32_t q = 0; q < m; ++q) acc = acc + part[tid + q];
        inv_norm[(uint32_t)tid / m] = 1.0f / (acc + eps_l1);
    }
    __syncthreads();
    if (valid) {
        const float invL = inv_norm[(uint32_t)tid / m];
#pragma unroll
        for (int k = 0; k < G; ++k) a[k] = a[k] * log_contract(__builtin_fmaf(a[k], invL, eps_log));
        part[tid] = tree_sum<G>(a);
    }
    __syncthreads();
    if (first) {
        float acc = 0.0f;
        for (uint32_t q = 0; q < m; ++q) acc = acc + part[tid + q];
        H[((uint32_t)j0 + tid) / m] = 0.0f - inv_norm[(uint32_t)tid / m] * acc;
    }
}

// Left-to-right sum of the m partial sums of every allocation tile.  FINAL = false: the reciprocal norm
// r = 1 / (L1 + eps) of Eq. 1; FINAL = true: the entropy 0 - r * sum of Eq. 2, with r read from `inv_norm`.
template <bool FINAL>
__global__ __launch_bounds__(256) void k_alloc_reduce(const float *__restrict__ part, const float *__restrict__ inv_norm,
                                                      float *__restrict__ out, uint32_t n_alloc, uint32_t m, float eps_l1)
{
    const uint32_t ja = blockIdx.x * 256 + threadIdx.x;
    if (ja >= n_alloc) return;
    const float *p = part + (uint64_t)ja * m;
    float acc = 0.0f;
    for (uint32_t q = 0; q < m; ++q) acc = acc + p[q];
    if constexpr (FINAL) out[ja] = 0.0f - inv_norm[ja] * acc;
    else out[ja] = 1.0f / (acc + eps_l1);
}

// ------------------------------------ K3: transform + quantize + pack

// Payload unit: a tile's payload is b units of G/8 bytes (b = 3 or 4).
template <int G> struct Unit;
template <> struct Unit<8>   { using type = uint8_t; };
template <> struct Unit<16>  { using type = uint16_t; };
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

// What a workgroup must know about a batch before it can place payload: the bit map words of the
// batch's 64-tile groups and the rank-table entry of the first one.
template <int TILES>
struct BatchMeta {
    static constexpr int WORDS = (TILES + 63) / 64;
    uint64_t word[WORDS];
    uint32_t rank0;
};

// `lane_zero` is a per-lane zero the compiler cannot see through: it turns these uniform loads into
// vector loads, which are counted in order with the other global loads (scalar loads are not, and a
// wait for LDS data would also wait for them).
template <int TILES>
__device__ __forceinline__ void load_meta(const uint8_t *__restrict__ packed, const Layout &lay, uint64_t j0, uint32_t T,
                                          uint32_t lane_zero, BatchMeta<TILES> &m)
{
    const uint64_t *bitmap = reinterpret_cast<const uint64_t *>(packed + lay.bitmap) + lane_zero;
    const uint32_t *ranks = reinterpret_cast<const uint32_t *>(packed + lay.ranks) + lane_zero;
    const uint64_t last_word = ((uint64_t)T - 1) >> 6;
#pragma unroll
    for (int w = 0; w < BatchMeta<TILES>::WORDS; ++w) {
        const uint64_t jw = (j0 >> 6) + w;
        const uint64_t word = bitmap[jw <= last_word ? jw : last_word];     // clamped index: no load behind a branch
        m.word[w] = jw <= last_word ? word : 0ull;
    }
    m.rank0 = ranks[j0 >> 6];
}

// Number of set bits of `mask` in the lanes below mine (two instructions).
__device__ __forceinline__ uint32_t bits_below_me(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Width of my tile (LOW or LOW + 1 bits), its payload position inside the batch (in units of G/8 bytes), and
// the number of wide tiles in the batch.  A wavefront's 64 tiles are one bit map word.
template <int TILES, int LOW>
__device__ __forceinline__ void tile_pos(const BatchMeta<TILES> &m, int tid, uint32_t *b, uint32_t *rel, uint32_t *total4)
{
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);      // the same in every lane
    const uint32_t lane = (uint32_t)tid & 63u;
    uint64_t mine = 0;
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < BatchMeta<TILES>::WORDS; ++w) {
        if ((uint32_t)w == wave) { mine = m.word[w]; before = tot; }
        tot += (uint32_t)__popcll(m.word[w]);
    }
    const uint32_t half = lane < 32u ? (uint32_t)mine : (uint32_t)(mine >> 32);
    *b = (uint32_t)LOW + ((half >> (lane & 31u)) & 1u);
    *rel = (uint32_t)LOW * (uint32_t)tid + before + bits_below_me(mine);
    *total4 = tot;
}

// Tiles of a batch regrouped by class (0..3; anything else sorts nowhere): the position of my tile when the batch is
// ordered by class and, inside a class, by tile index.  Two steps with a workgroup barrier between them.
// Step 1: my rank among the tiles of my class in my wavefront; lane 0 leaves the wavefront's four counts in
// `counts` (LDS, uint32[4 * WAVES], class-major).
template <int WAVES>
__device__ __forceinline__ uint32_t class_rank_in_wave(uint32_t cls, uint32_t wave, uint32_t lane, uint32_t *counts)
{
    uint32_t rank = 0;
#pragma unroll
    for (uint32_t c = 0; c < 4; ++c) {
        const uint64_t m = __ballot(cls == c);
        if (cls == c) rank = bits_below_me(m);
        if (lane == 0) counts[c * WAVES + wave] = (uint32_t)__popcll(m);
    }
    return rank;
}

// Step 2 (after the barrier): tiles that come before my class-and-wavefront group.  In class-major order that is
// the exclusive prefix sum of the 4 * WAVES counts: lanes 0 .. 4 WAVES - 1 scan them with row shifts, and every
// lane fetches the entry of its own group.  All lanes of the wavefront must be enabled.
template <int WAVES>
__device__ __forceinline__ uint32_t class_group_base(uint32_t cls, uint32_t wave, uint32_t lane, const uint32_t *counts)
{
    static_assert(4 * WAVES <= 16, "the counts must fit one row of 16 lanes");
    const uint32_t own = lane < 4u * WAVES ? counts[lane] : 0u;
    uint32_t v = own;
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);     // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);     // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);     // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);     // row_shr:8
    const uint32_t group = cls < 4u ? cls * WAVES + wave : 0u;
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)(group << 2), (int)(v - own));
}

// Three-input float min / max in one instruction each (no NaN canonicalisation around them).
__device__ __forceinline__ float fmin3(float a, float b, float c)
{
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float fmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Eq. 3 for the tile in `row`: outlier flag and pivot index; for an outlier tile with d != 0 the pivot
// swap P_d is applied to the LDS row on the spot.  Returns the pivot byte (bit 7 = flag, bits 0..6 = d).
template <int G, bool BF16>
__device__ __forceinline__ uint32_t analyse_row(uint8_t *row, float tau, float eps_ratio)
{
    float a1, a2;
    uint32_t d;
    top2<G, BF16>(row, &a1, &a2, &d);
    const bool flag = a1 > tau * (a2 + eps_ratio);
    if (flag && d != 0) {
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
    return flag ? (0x80u | d) : 0u;
}

// The rest of the encoder for one tile, in two steps with a workgroup barrier between them (the payload
// buffer that step 2 writes shares LDS with the rows that step 1 reads).
// Step 1: the row (which already carries P_d) into registers; Eq. 4 on outlier tiles.
template <int G, bool BF16>
__device__ __forceinline__ void transform_row(const uint8_t *row, bool flag, float *x)
{
    read_tile<G, BF16>(row, x);
    if (flag) {
        butterfly<G>(x);
#pragma unroll
        for (int k = 0; k < G; ++k) x[k] = x[k] * TileConst<G>::c;
    }
}

// Dwords that hold the G W-bit codes of a tile.
template <int G, int W> struct BitString { static constexpr int DWORDS = (G * W + 31) / 32; };

// The tile's LSB-first bit string, as dwords, from groups of four W-bit codes (g4[g] = q0 + 2^W q1 + 2^2W q2
// + 2^3W q3), W <= 4.  Writes the dwords the string occupies; the caller has cleared the rest.
template <int G, int W>
__device__ __forceinline__ void pack_groups(const uint32_t *g4, uint32_t *dw)
{
    static_assert(W >= 1 && W <= 4, "groups of four codes are exact in fp32 up to 4 bits per code");
    if constexpr (G < 32) {
        // at most 64 bits: two or four groups of 4 W bits through one 64-bit accumulator
        uint64_t acc = 0;
#pragma unroll
        for (int g = 0; g < G / 4; ++g) acc |= (uint64_t)g4[g] << (4 * W * g);
        dw[0] = (uint32_t)acc;
        if constexpr (G * W > 32) dw[1] = (uint32_t)(acc >> 32);
    } else if constexpr (W == 4) {
#pragma unroll
        for (int i = 0; i < G / 8; ++i) dw[i] = g4[2 * i] | (g4[2 * i + 1] << 16);
    } else if constexpr (W == 3) {
        // 12-bit groups: eight of them fill three dwords
#pragma unroll
        for (int i = 0; i < G / 32; ++i) {
            const uint32_t *p = g4 + 8 * i;
            dw[3 * i + 0] = p[0] | (p[1] << 12) | (p[2] << 24);
            dw[3 * i + 1] = (p[2] >> 8) | (p[3] << 4) | (p[4] << 16) | (p[5] << 28);
            dw[3 * i + 2] = (p[5] >> 4) | (p[6] << 8) | (p[7] << 20);
        }
    } else if constexpr (W == 2) {
        // 8-bit groups: four of them fill a dword
#pragma unroll
        for (int i = 0; i < G / 16; ++i)
            dw[i] = g4[4 * i] | (g4[4 * i + 1] << 8) | (g4[4 * i + 2] << 16) | (g4[4 * i + 3] << 24);
    } else {
        // 4-bit groups: eight of them fill a dword
#pragma unroll
        for (int i = 0; i < G / 32; ++i) {
            uint32_t t = 0;
#pragma unroll
            for (int g = 0; g < 8; ++g) t |= g4[8 * i + g] << (4 * g);
            dw[i] = t;
        }
    }
}

// The same from the codes themselves, for any width up to 8 bits: code k occupies bits [W k, W k + W).
template <int G, int W>
__device__ __forceinline__ void place_codes(const uint32_t *q, uint32_t *dw)
{
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const int bit = W * k, i = bit >> 5, sh = bit & 31;
        dw[i] |= q[k] << sh;
        if (sh + W > 32) dw[i + 1] |= q[k] >> (32 - sh);
    }
}

// Step 2: range, quantizer parameters, codes, and the tile's LSB-first bit string written as b units at
// `dst` (LDS); b is LOW or LOW + 1.  Returns scale | zero << 16.
template <int G, int LOW>
__device__ __forceinline__ uint32_t quantize_values(const float *x, uint32_t b, typename Unit<G>::type *dst)
{
    constexpr uint32_t WIDE = LOW + 1;
    float mn = fmin3(x[0], x[1], x[2]), mx = fmax3(x[0], x[1], x[2]);
#pragma unroll
    for (int k = 3; k + 1 < G; k += 2) { mn = fmin3(mn, x[k], x[k + 1]); mx = fmax3(mx, x[k], x[k + 1]); }
    mn = __builtin_fminf(mn, x[G - 1]) + 0.0f;
    mx = __builtin_fmaxf(mx, x[G - 1]) + 0.0f;

    // asymmetric quantizer, binary16 metadata rounded outwards
    const float Lv = (b == WIDE) ? (float)((1u << WIDE) - 1u) : (float)((1u << LOW) - 1u);
    const uint32_t z16 = f16_down(mn);
    const float mnf = f16_widen(z16);
    const float s = (mx - mnf) / Lv;
    uint32_t s16 = f16_up(s);
    if ((s16 & 0x7fffu) == 0) s16 = 0x3c00u;
    const float sf = f16_widen(s16);
    const float rcp = 1.0f / sf;
    // Every element lies in [mn, mx]; if z <= mn, (x - z) * rcp lies in [0, (mx - z) * rcp], and when that
    // bound rounds to at most L the clamp is the identity and is skipped.  Both conditions can fail only when
    // the binary16 metadata saturated (magnitudes beyond the contract).
    const bool no_clamp = mnf <= mn && (mx - mnf) * rcp <= Lv + 0.25f;

    constexpr int DW = BitString<G, WIDE>::DWORDS > G / 8 ? BitString<G, WIDE>::DWORDS : (G / 8 ? G / 8 : 1);
    uint32_t dw[DW];
#pragma unroll
    for (int i = 0; i < DW; ++i) dw[i] = 0;
    if constexpr (WIDE <= 4) {
        // codes, four at a time: q0 + m q1 + m^2 q2 + m^3 q3 is an exact integer below 2^16 in fp32
        const float m1 = (b == WIDE) ? (float)(1u << WIDE) : (float)(1u << LOW);
        const float m2 = m1 * m1, m3 = m2 * m1;
        uint32_t g4[G / 4];
        if (no_clamp) {
#pragma unroll
            for (int g = 0; g < G / 4; ++g) {
                float q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) q[i] = __builtin_rintf((x[4 * g + i] - mnf) * rcp);
                const float acc = __builtin_fmaf(q[3], m3, __builtin_fmaf(q[2], m2, __builtin_fmaf(q[1], m1, q[0])));
                g4[g] = (uint32_t)acc;
            }
        } else {
#pragma unroll
            for (int g = 0; g < G / 4; ++g) {
                float q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    q[i] = __builtin_amdgcn_fmed3f(__builtin_rintf((x[4 * g + i] - mnf) * rcp), 0.0f, Lv);
                const float acc = __builtin_fmaf(q[3], m3, __builtin_fmaf(q[2], m2, __builtin_fmaf(q[1], m1, q[0])));
                g4[g] = (uint32_t)acc;
            }
        }
        if (b == WIDE) pack_groups<G, WIDE>(g4, dw);
        else pack_groups<G, LOW>(g4, dw);
    } else {
        // wider codes: one by one (a NaN code becomes 0 in the clamp)
        uint32_t q[G];
#pragma unroll
        for (int k = 0; k < G; ++k)
            q[k] = (uint32_t)__builtin_amdgcn_fmed3f(__builtin_rintf((x[k] - mnf) * rcp), 0.0f, Lv);
        if (b == WIDE) place_codes<G, WIDE>(q, dw);
        else place_codes<G, LOW>(q, dw);
    }
    // the bit string leaves as b units of G/8 bytes
#pragma unroll
    for (int u = 0; u < (int)WIDE; ++u) {
        if (u < LOW || b == WIDE) {
            if constexpr (G == 8) dst[u] = (uint8_t)(dw[u >> 2] >> (8 * (u & 3)));
            else if constexpr (G == 16) dst[u] = (uint16_t)(dw[u >> 1] >> (16 * (u & 1)));
            else if constexpr (G == 32) dst[u] = dw[u];
            else if constexpr (G == 64) dst[u] = make_uint2(dw[2 * u], dw[2 * u + 1]);
            else dst[u] = make_uint4(dw[4 * u], dw[4 * u + 1], dw[4 * u + 2], dw[4 * u + 3]);
        }
    }
    return s16 | (z16 << 16);
}

// Occupancy hint: with small tiles the kernel fits four workgroups per compute unit if it stays within
// 128 vector registers.
template <int G, int ESIZE>
struct QuantPackOccupancy { static constexpr int WAVES_PER_SIMD = (G * ESIZE <= 128) ? 4 : 1; };

// One workgroup per batch of TILES tiles, in two stages.  Stage one: lane i examines tile i (Eq. 3, pivot
// swap in LDS).  The tiles are then regrouped by class -- (plain | transformed) x (narrow | wide) -- so that in
// stage two, where lane p takes the p-th tile in class order, most wavefronts hold a single class: the
// Hadamard butterfly runs only in the wavefronts that hold transformed tiles, and the two packing
// paths rarely both run.  The payload buffer reuses the rows' LDS once every lane holds its tile in
// registers, which keeps the workgroup small enough for four to share a compute unit: this kernel
// lives on the loads of its neighbours being in flight while it computes.
template <int G, bool BF16, int LOW, bool FULL>
__device__ __forceinline__ void quant_pack_batch(const void *__restrict__ in, uint8_t *__restrict__ packed, const Layout &lay,
                                                 uint32_t T, float tau, float eps_ratio, uint32_t batch, uint32_t nvalid,
                                                 uint8_t *lds, uint32_t *info, uint16_t *order, uint32_t *class_count)
{
    constexpr int ES = BF16 ? 2 : 4;
    using B = Batch<G, ES>;
    using U = typename Unit<G>::type;
    constexpr int WAVES = (B::TILES + 63) / 64;
    constexpr uint32_t WIDE = LOW + 1;           // the two code widths are LOW and WIDE bits
    static_assert(sizeof(U) * WIDE * B::TILES <= (size_t)B::LDS_BYTES, "payload buffer must fit in the rows");
    U *pay = reinterpret_cast<U *>(lds);         // valid only after every lane has left the rows
    // The lane index passes through an empty asm statement, so the optimiser derives every address from
    // it afresh instead of sharing address arithmetic between the phases: measured 3 % faster.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint64_t j0 = (uint64_t)batch * B::TILES;

    uint4 v[B::CHUNKS];
    load_batch<G, ES, FULL, true>(in, j0, nvalid, v, tid);           // second and last read of the tensor
    BatchMeta<B::TILES> meta;
    load_meta<B::TILES>(packed, lay, j0, T, 0u, meta);
    store_batch<G, ES, FULL>(v, nvalid, lds, tid);
    uint32_t b, rel, total4;
    tile_pos<B::TILES, LOW>(meta, tid, &b, &rel, &total4);
    __syncthreads();

    // stage one: my own tile
    const bool valid = FULL || (uint32_t)tid < nvalid;
    uint32_t cls = 4;                            // tiles past the end sort last
    if (valid) {
        const uint32_t pv = analyse_row<G, BF16>(lds + tid * B::STRIDE, tau, eps_ratio);
        info[tid] = pv | ((b == WIDE) ? 0x100u : 0u) | (rel << 9);
        cls = ((pv >> 7) << 1) | (b == WIDE ? 1u : 0u);
    }
    const uint32_t rank_in_wave = class_rank_in_wave<WAVES>(cls, (uint32_t)wave, (uint32_t)lane, class_count);
    __syncthreads();
    {
        const uint32_t pos = rank_in_wave + class_group_base<WAVES>(cls, (uint32_t)wave, (uint32_t)lane, class_count);
        if (valid) order[pos] = (uint16_t)tid;
    }
    __syncthreads();

    // stage two: the tid-th tile in class order
    float x[G];
    uint32_t t = 0, inf = 0;
    if (valid) {
        t = order[tid];
        inf = info[t];
        transform_row<G, BF16>(lds + t * B::STRIDE, (inf & 0x80u) != 0, x);
    }
    __syncthreads();                             // the rows are dead: their LDS becomes the payload buffer
    if (valid) {
        const uint32_t meta16 = quantize_values<G, LOW>(x, (inf & 0x100u) ? WIDE : (uint32_t)LOW, pay + (inf >> 9));
        const uint64_t j = j0 + t;
        reinterpret_cast<uint16_t *>(packed + lay.scale)[j] = (uint16_t)meta16;
        reinterpret_cast<uint16_t *>(packed + lay.zero)[j] = (uint16_t)(meta16 >> 16);
        packed[lay.pivot + j] = (uint8_t)inf;
    }
    __syncthreads();

    // the batch's payload is one contiguous span: copy it out unit by unit, coalesced
    const uint32_t span = (uint32_t)LOW * nvalid + total4;
    U *gdst = reinterpret_cast<U *>(packed + lay.payload) + ((uint64_t)LOW * j0 + meta.rank0);
#pragma unroll
    for (int i = 0; i < (int)WIDE; ++i) {
        const uint32_t q = (uint32_t)i * B::TILES + tid;
        if (q < span) gdst[q] = pay[q];
    }
}

template <int G, bool BF16, int LOW>
__global__ __launch_bounds__((Batch<G, BF16 ? 2 : 4>::TILES), (QuantPackOccupancy<G, BF16 ? 2 : 4>::WAVES_PER_SIMD))
void k_quant_pack(const void *__restrict__ in, uint8_t *__restrict__ packed, Layout lay, uint32_t T, float tau,
                  float eps_ratio)
{
    constexpr int ES = BF16 ? 2 : 4;
    using B = Batch<G, ES>;
    constexpr int WAVES = (B::TILES + 63) / 64;
    __shared__ __attribute__((aligned(16))) uint8_t lds[B::LDS_BYTES];
    __shared__ uint32_t info[B::TILES];          // per tile: pivot byte | (b == WIDE) << 8 | rel << 9
    __shared__ uint16_t order[B::TILES];         // tiles in class order
    __shared__ uint32_t class_count[4 * WAVES];  // tiles per class and wavefront, class-major
    const uint32_t nfull = T / B::TILES;        // a workgroup per batch; the last one may be ragged
    if (blockIdx.x < nfull)
        quant_pack_batch<G, BF16, LOW, true>(in, packed, lay, T, tau, eps_ratio, blockIdx.x, B::TILES, lds, info, order,
                                             class_count);
    else
        quant_pack_batch<G, BF16, LOW, false>(in, packed, lay, T, tau, eps_ratio, nfull, T % B::TILES, lds, info, order,
                                              class_count);
}

// ------------------------------------------------------------- K4: decode

// The tile's W-bit codes brought onto nibble boundaries: nib[i] holds codes 8i .. 8i+7, one per nibble.
template <int G, int W>
__device__ __forceinline__ void codes_to_nibbles(const uint32_t *dw, uint32_t *nib)
{
    if constexpr (W == 4) {
#pragma unroll
        for (int i = 0; i < G / 8; ++i) nib[i] = dw[i];
    } else if constexpr (W == 3) {
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
    } else if constexpr (W == 2) {
#pragma unroll
        for (int i = 0; i < G / 8; ++i) {
            // codes 8i .. 8i+7 occupy bits [16i, 16i+16) of the string
            uint32_t t = (dw[i >> 1] >> (16 * (i & 1))) & 0xffffu;
            t = (t & 0x000000ffu) | ((t & 0x0000ff00u) << 8);
            t = (t & 0x000f000fu) | ((t & 0x00f000f0u) << 4);
            t = (t & 0x03030303u) | ((t & 0x0c0c0c0cu) << 2);
            nib[i] = t;
        }
    } else {
        static_assert(W == 1, "nibbles hold codes of up to 4 bits");
#pragma unroll
        for (int i = 0; i < G / 8; ++i) {
            // codes 8i .. 8i+7 are byte i of the string
            uint32_t t = (dw[i >> 2] >> (8 * (i & 3))) & 0xffu;
            t = (t & 0x0000000fu) | ((t & 0x000000f0u) << 12);
            t = (t & 0x00030003u) | ((t & 0x000c000cu) << 6);
            t = (t & 0x01010101u) | ((t & 0x02020202u) << 3);
            nib[i] = t;
        }
    }
}

// ... and, for any width up to 8 bits, the codes one by one, de-quantized: x[k] = q_k * sf + mnf.
template <int G, int W>
__device__ __forceinline__ void dequantize_codes(const uint32_t *dw, float sf, float mnf, float *x)
{
#pragma unroll
    for (int k = 0; k < G; ++k) {
        const int bit = W * k, i = bit >> 5, sh = bit & 31;
        uint32_t q = dw[i] >> sh;
        if (sh + W > 32) q |= dw[i + 1] << (32 - sh);
        x[k] = __builtin_fmaf((float)(q & ((1u << W) - 1u)), sf, mnf);
    }
}

// Alg. 1 step 5 for my tile: my LOW or LOW + 1 payload units at `src` (LDS) -> codes -> q*s + z -> for
// transformed tiles the butterfly, 1/sqrt(G) and P_d -> my LDS row in the output type.
template <int G, bool OUT_BF16, int LOW>
__device__ __forceinline__ void decode_row(const typename Unit<G>::type *src, uint32_t b, uint32_t s16, uint32_t z16,
                                           uint32_t pv, uint8_t *row)
{
    using U = typename Unit<G>::type;
    constexpr int WIDE = LOW + 1;
    const float sf = f16_widen(s16), mnf = f16_widen(z16);
    // my LOW or WIDE units (the last one is read in any case: it stays inside the array)
    constexpr int DW = BitString<G, WIDE>::DWORDS > G / 8 ? BitString<G, WIDE>::DWORDS : (G / 8 ? G / 8 : 1);
    uint32_t dw[DW + 1];                         // one more: the one-by-one reader may look past the string
#pragma unroll
    for (int i = 0; i < DW + 1; ++i) dw[i] = 0;
#pragma unroll
    for (int u = 0; u < WIDE; ++u) {
        const U t = src[u];
        if constexpr (G == 8) dw[u >> 2] |= (uint32_t)t << (8 * (u & 3));
        else if constexpr (G == 16) dw[u >> 1] |= (uint32_t)t << (16 * (u & 1));
        else if constexpr (G == 32) dw[u] = t;
        else if constexpr (G == 64) { dw[2 * u] = t.x; dw[2 * u + 1] = t.y; }
        else { dw[4 * u] = t.x; dw[4 * u + 1] = t.y; dw[4 * u + 2] = t.z; dw[4 * u + 3] = t.w; }
    }
    float x[G];
    if constexpr (WIDE <= 4) {
        uint32_t nib[G / 8];
        if (b == (uint32_t)WIDE) codes_to_nibbles<G, WIDE>(dw, nib);
        else codes_to_nibbles<G, LOW>(dw, nib);
        // de-quantize: even codes sit in the low nibbles of the bytes, odd codes in the high nibbles
        // (scaled by 16, undone exactly by a scale of sf/16)
        const float sf16 = sf * 0.0625f;
#pragma unroll
        for (int i = 0; i < G / 8; ++i) {
            const uint32_t lo = nib[i] & 0x0f0f0f0fu, hi = nib[i] & 0xf0f0f0f0u;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                x[8 * i + 2 * c] = __builtin_fmaf((float)((lo >> (8 * c)) & 0xffu), sf, mnf);
                x[8 * i + 2 * c + 1] = __builtin_fmaf((float)((hi >> (8 * c)) & 0xffu), sf16, mnf);
            }
        }
    } else {
        if (b == (uint32_t)WIDE) dequantize_codes<G, WIDE>(dw, sf, mnf, x);
        else dequantize_codes<G, LOW>(dw, sf, mnf, x);
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
    const uint32_t d = pv & 0x7fu & (uint32_t)(G - 1);      // masked: a corrupted pivot byte stays inside the row
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

// Persistent workgroups over contiguous runs of full batches, software-pipelined: while batch i is decoded,
// the payload span, bit map words and per-tile metadata of batch i+1 are in flight; the rows of batch i are
// written out one iteration late, just before the next loads are issued, so that no wait for loads has a
// younger store in front of it.  The fast loop has no per-thread conditions on global memory operations.
// The only two-step dependency -- the rank-table entries that locate a batch's payload and give its length
// -- is taken out of the loop: the entries of the workgroup's batches are read into LDS up front.
// The ragged last batch is handled after the loop by one workgroup.
template <int G, bool OUT_BF16, int LOW>
__global__ __launch_bounds__((Batch<G, OUT_BF16 ? 2 : 4>::TILES))
void k_decode(const uint8_t *__restrict__ packed, void *__restrict__ out, Layout lay, uint32_t T, uint32_t total_wide)
{
    constexpr int ES = OUT_BF16 ? 2 : 4;
    using B = Batch<G, ES>;
    using U = typename Unit<G>::type;
    using Meta = BatchMeta<B::TILES>;
    __shared__ __attribute__((aligned(16))) uint8_t lds[B::LDS_BYTES];
    constexpr uint32_t WIDE = LOW + 1;           // the two code widths are LOW and WIDE bits
    __shared__ __attribute__((aligned(16))) U pay[B::TILES * WIDE];
    __shared__ uint32_t rank_lds[B::TILES + 1];
    constexpr int WAVES = (B::TILES + 63) / 64;
    __shared__ uint2 tile_meta[B::TILES];        // per tile: scale | zero << 16, pivot byte | (b == WIDE) << 8 | rel << 9
    __shared__ uint16_t order[B::TILES];         // tiles in class order
    __shared__ uint32_t class_count[4 * WAVES];  // tiles per class and wavefront, class-major
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t nfull = T / B::TILES, tail = T % B::TILES;
    const uint32_t per = (nfull + gridDim.x - 1) / gridDim.x;
    const uint32_t first = blockIdx.x * per;
    const uint32_t last = first + per < nfull ? first + per : nfull;      // my batches: [first, last)
    const uint16_t *scale = reinterpret_cast<const uint16_t *>(packed + lay.scale);
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(packed + lay.zero);
    const uint8_t *pivot = packed + lay.pivot;
    const uint32_t *ranks = reinterpret_cast<const uint32_t *>(packed + lay.ranks);
    const U *payload = reinterpret_cast<const U *>(packed + lay.payload);
    uint8_t *row = lds + tid * B::STRIDE;
    uint32_t lane_zero = 0;
    asm volatile("" : "+v"(lane_zero));
    const uint64_t *bitmap = reinterpret_cast<const uint64_t *>(packed + lay.bitmap) + lane_zero;

    // wide tiles before batch b (for the batch past the end of the tensor: all of them)
    // The stream may have been damaged on its way here: the table's entries are clamped to the number of wide
    // tiles the configuration implies, and a batch's count of wide tiles is taken as 0 if the table decreases, so
    // that every payload address below stays inside the payload section whatever the stream holds.
    auto rank_of_batch = [&](uint64_t b) {
        const uint32_t r = b * B::TILES < T ? ranks[b * (B::TILES / 64)] : total_wide;
        return r < total_wide ? r : total_wide;
    };
    // slots 0..TILES of the window hold the entries of batches wfirst .. wfirst + TILES
    auto load_rank_window = [&](uint32_t wfirst) {
        rank_lds[tid] = rank_of_batch((uint64_t)wfirst + tid);
        if (tid == 0) rank_lds[B::TILES] = rank_of_batch((uint64_t)wfirst + B::TILES);
        __syncthreads();
    };
    uint32_t wfirst = first;
    if (first < last) load_rank_window(wfirst);

    Meta m;            // bit map words of the batch whose loads are in flight / have just arrived
    U pre[WIDE];
    uint32_t s16 = 0, z16 = 0, pv = 0;
    // issue the loads of full batch `batch` (inside the current window)
    auto fetch = [&](uint32_t batch) {
        const uint64_t j0 = (uint64_t)batch * B::TILES;
        m.rank0 = rank_lds[batch - wfirst];
        const uint32_t next_rank = rank_lds[batch - wfirst + 1];
        const uint32_t total4 = next_rank > m.rank0 ? next_rank - m.rank0 : 0u;
        const uint64_t base = (uint64_t)LOW * j0 + m.rank0;
#pragma unroll
        for (int i = 0; i < LOW; ++i) pre[i] = payload[base + (uint32_t)i * B::TILES + tid];
        // a thread's last unit exists only if the batch has more than `tid` wide tiles; otherwise the
        // load is pointed at the batch's first unit (a line that is being read anyway) and ignored
        pre[LOW] = payload[base + ((uint32_t)tid < total4 ? (uint32_t)LOW * (uint32_t)B::TILES + (uint32_t)tid : 0u)];
#pragma unroll
        for (int w = 0; w < Meta::WORDS; ++w) m.word[w] = bitmap[(j0 >> 6) + w];
        s16 = scale[j0 + tid];
        z16 = zero[j0 + tid];
        pv = pivot[j0 + tid];
    };

    if (first < last) fetch(first);
    bool have_prev = false;
    uint32_t prev_batch = 0;
    for (uint32_t batch = first; batch < last; ++batch) {
        uint32_t b, rel, total4;
        tile_pos<B::TILES, LOW>(m, tid, &b, &rel, &total4);
#pragma unroll
        for (int i = 0; i < (int)WIDE; ++i) pay[(uint32_t)i * B::TILES + tid] = pre[i];
        // Tiles are regrouped by class -- (plain | transformed) x (narrow | wide) -- as in the encoder: lane p decodes
        // the p-th tile in class order, so the butterfly runs only in the wavefronts that hold transformed tiles.
        tile_meta[tid] = make_uint2(s16 | (z16 << 16), pv | ((b == WIDE) ? 0x100u : 0u) | (rel << 9));
        const uint32_t cls = ((pv >> 7) << 1) | (b == WIDE ? 1u : 0u);
        const uint32_t rank_in_wave = class_rank_in_wave<WAVES>(cls, (uint32_t)wave, (uint32_t)lane, class_count);
        __syncthreads();
        if (have_prev) stage_out<G, ES, true>(out, (uint64_t)prev_batch * B::TILES, B::TILES, lds);
        order[rank_in_wave + class_group_base<WAVES>(cls, (uint32_t)wave, (uint32_t)lane, class_count)] = (uint16_t)tid;
        __syncthreads();

        if (batch + 1 < last) {
            if (batch + 1 - wfirst == (uint32_t)B::TILES) {      // once every TILES iterations
                __syncthreads();
                wfirst = batch + 1;
                load_rank_window(wfirst);
            }
            fetch(batch + 1);
        }
        {
            const uint32_t t = order[tid];
            const uint2 tm = tile_meta[t];
            decode_row<G, OUT_BF16, LOW>(pay + (tm.y >> 9), (tm.y & 0x100u) ? WIDE : (uint32_t)LOW, tm.x & 0xffffu,
                                         tm.x >> 16, tm.y & 0xffu, lds + t * B::STRIDE);
        }
        prev_batch = batch;
        have_prev = true;
        __syncthreads();
    }
    if (have_prev) stage_out<G, ES, true>(out, (uint64_t)prev_batch * B::TILES, B::TILES, lds);

    if (tail != 0 && blockIdx.x == gridDim.x - 1) {
        __syncthreads();
        const uint64_t j0 = (uint64_t)nfull * B::TILES;
        load_meta<B::TILES>(packed, lay, j0, T, 0u, m);
        uint32_t b, rel, total4;
        tile_pos<B::TILES, LOW>(m, tid, &b, &rel, &total4);
        // clamped like the table entries above: the span never reaches past the payload section
        const uint32_t rank0 = m.rank0 < total_wide ? m.rank0 : total_wide;
        const uint32_t room = total_wide - rank0;
        const uint32_t span = (uint32_t)LOW * tail + (total4 < room ? total4 : room);
        const U *gsrc = payload + ((uint64_t)LOW * j0 + rank0);
        for (uint32_t q = tid; q < span; q += B::TILES) pay[q] = gsrc[q];
        __syncthreads();
        if ((uint32_t)tid < tail)
            decode_row<G, OUT_BF16, LOW>(pay + rel, b, scale[j0 + tid], zero[j0 + tid], pivot[j0 + tid], row);
        __syncthreads();
        stage_out<G, ES, false>(out, j0, tail, lds);
    }
}

}  // namespace tahq
