// Top-p% tile selection (Sec. 3.2): inside every ranking unit the k (allocation) tiles of highest entropy get
// the wider code (4 bits by default), ties going to the lower tile index.  Exact, deterministic, no sort.
// Entropies map to order-preserving 32-bit keys; three ways to find the k-th largest key K*, how many tiles equal to
// K* are still wanted (`take`), and from them the bit map and the rank table:
//
//   * ranking units of at most 32768 tiles: k_select_small, one workgroup per unit in one launch (keys in registers,
//     radix passes on an LDS histogram), because at that size several launches cost more than the work;
//   * larger units that start on 64-tile boundaries and are whole batches of the entropy kernel: that kernel also
//     counts the entropies over 2048 linear bins per unit; k_select_classify settles every tile outside the bin that
//     holds K* and lists the tiles inside it, k_select_resolve ranks that list (further down in this file);
//   * everything else, and every unit when the caller forces it: three histogram passes (10 + 11 + 11 bits, from the
//     top; the first one folded into the entropy kernel where units are whole batches) find K* and `take`; then, per
//     segment of tiles, counts of keys == K* and > K*, whose prefix sums give every tile its place among the equal keys
//     (index order) and every 64-tile group its rank-table entry: k_radix_pass x 2, k_seg_count, k_assign.
//
// Kernels never wait on each other inside a launch: every dependency is a launch boundary, and the
// small reductions a later kernel needs (which bin holds the k-th key, prefix over segments) are
// recomputed by every block from a few KB of global data.
//
// In the third way the histograms of digits 1 and 2 are kept in two levels so that no address takes more than a handful
// of global atomics: every workgroup stores its own 2048-bin histogram with plain stores and adds only the
// totals of its 64 super-bins (32 bins each) atomically.  The reader picks the super-bin from the 64
// totals, then sums the workgroups' counts for the 32 bins inside it.
#pragma once
#include "tahq_common.hpp"
#include "tahq_stream_kernels.hpp"

namespace tahq {

// Inclusive scan over the 64 lanes of a wavefront with data-parallel-primitive moves (all lanes must be
// enabled): shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0 / 2 is added to
// row 1 / 3, then the last lane of the lower half to the upper half.  A lane without a source adds 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    v += dpp_or_zero<0x111, 0xF>(v);     // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);     // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);     // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);     // row_shr:8
    v += dpp_or_zero<0x142, 0xA>(v);     // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xC>(v);     // row_bcast:31 into rows 2 and 3
    return v;
}

// selection state of one ranking unit (uint32[8] in the workspace)
enum { ST_BIN0 = 0, ST_BIN1 = 1, ST_BIN2 = 2, ST_KREM0 = 3, ST_KREM1 = 4, ST_KEY = 5, ST_TAKE = 6 };

// Which bin of a BINS-bin histogram holds the `want`-th largest key (bins counted from the top), and how
// many keys are still wanted inside that bin.  Run by one full wavefront; lane l owns the BINS/64 bins
// just below BINS - l*BINS/64.  Result is returned in every lane.
template <int BINS>
__device__ __forceinline__ void pick_bin(const uint32_t *__restrict__ hist, uint32_t want, uint32_t *bin,
                                         uint32_t *rem)
{
    constexpr int PER = BINS / 64;
    const int lane = threadIdx.x & 63;
    uint32_t c[PER], mine = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) { c[i] = hist[BINS - 1 - (lane * PER + i)]; mine += c[i]; }
    uint32_t above = wave_incl_scan(mine) - mine;      // keys in bins above mine
    uint32_t found_bin = 0, found_rem = 0;
    bool found = false;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        if (!found && above < want && want <= above + c[i]) {
            found = true;
            found_bin = BINS - 1 - (lane * PER + i);
            found_rem = want - above;
        }
        above += c[i];
    }
    // exactly one lane finds it when 1 <= want <= total; otherwise fall back to bin 0 / 0 wanted
    const uint64_t who = __ballot(found);
    const int src = who ? (int)__ffsll((unsigned long long)who) - 1 : 0;
    *bin = (uint32_t)__shfl((int)found_bin, src, 64);
    *rem = (uint32_t)__shfl((int)found_rem, src, 64);
}

// Two-level variant of pick_bin for digits 1 and 2: `coarse` holds the 64 super-bin totals, `partial` the
// `hb` per-workgroup histograms.  Run by one full wavefront; result in every lane.
__device__ __forceinline__ void pick_bin_two_level(const uint32_t *__restrict__ coarse,
                                                   const uint32_t *__restrict__ partial, uint32_t hb, uint32_t want,
                                                   uint32_t *bin, uint32_t *rem)
{
    const int lane = threadIdx.x & 63;
    // super-bins from the top: lane l looks at super-bin 63 - l
    const uint32_t c = coarse[63 - lane];
    const uint32_t above = wave_incl_scan(c) - c;
    const bool hit = above < want && want <= above + c;
    const uint64_t who = __ballot(hit);
    const int src = who ? (int)__ffsll((unsigned long long)who) - 1 : 0;
    const uint32_t sb = 63u - (uint32_t)src;
    const uint32_t want2 = want - (uint32_t)__shfl((int)above, src, 64);
    // the 32 bins of that super-bin, from the top: lanes l and l+32 split the workgroups of bin 31 - (l & 31)
    const uint32_t b_in = 31u - ((uint32_t)lane & 31u);
    // (all loads first, then the sum: a rolled loop would pay one memory latency per workgroup)
    uint32_t part[32];
#pragma unroll
    for (uint32_t i = 0; i < 32; ++i) {
        const uint32_t blk = ((uint32_t)lane >> 5) + 2 * i;
        part[i] = partial[(uint64_t)(blk < hb ? blk : 0u) * kHistBins + sb * 32 + b_in];    // clamped, not branched
    }
    uint32_t sum = 0;
#pragma unroll
    for (uint32_t i = 0; i < 32; ++i) sum += (((uint32_t)lane >> 5) + 2 * i) < hb ? part[i] : 0u;
    sum += (uint32_t)__shfl_xor((int)sum, 32, 64);
    const uint32_t mine = lane < 32 ? sum : 0u;
    const uint32_t above2 = wave_incl_scan(mine) - mine;
    const bool hit2 = lane < 32 && above2 < want2 && want2 <= above2 + mine;
    const uint64_t who2 = __ballot(hit2);
    const int src2 = who2 ? (int)__ffsll((unsigned long long)who2) - 1 : 0;
    *bin = sb * 32 + (31u - (uint32_t)src2);
    *rem = want2 - (uint32_t)__shfl((int)above2, src2, 64);
}

// One radix pass.  Digits: pass 0 = key bits 31..22 (1024 bins), pass 1 = bits 21..11, pass 2 = bits 10..0
// (2048 bins each).  Pass p > 0 first derives, from the histogram of pass p-1, the bin chosen there (every
// block does this; block 0 of the unit also records it in `state`), then histograms digit p of the keys
// whose higher digits match.  Pass 0 runs as a kernel of its own only when the entropy kernel could not
// build its histogram; PEEL > 0 then aggregates equal digits inside a wavefront before touching LDS
// (it sees only a handful of distinct digits, which would serialize the LDS atomics).
template <int PASS, int PEEL>
__global__ __launch_bounds__(256) void k_radix_pass(const float *__restrict__ H, uint32_t n, uint32_t k,
                                                    uint32_t *__restrict__ hist0, uint32_t *__restrict__ coarse,
                                                    uint32_t *__restrict__ partial, uint32_t *__restrict__ state)
{
    constexpr int BINS = PASS == 0 ? (int)kDigit0Bins : (int)kHistBins;
    __shared__ uint32_t lh[BINS];
    __shared__ uint32_t chosen[2];
    const uint32_t u = blockIdx.y, hb = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t *ust = state + (uint64_t)u * 8;
    const float *uH = H + (uint64_t)u * n;
    uint32_t *ucoarse = coarse + (uint64_t)u * 2 * 64;                    // [2][64]
    uint32_t *upartial = partial + (uint64_t)u * 2 * hb * kHistBins;      // [2][hb][2048]

    for (int i = tid; i < BINS; i += 256) lh[i] = 0;

    // every thread walks the unit's keys in steps of the grid, sixteen loads in flight at a time; the first
    // sixteen are issued before the bin of the previous pass is worked out, which they do not depend on.
    // All loads use a clamped index: a load behind a branch would wait for the one before it.
    constexpr int R = 16;
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    const uint64_t base0 = (uint64_t)blockIdx.x * 256 + tid;
    float h[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint64_t i = base0 + r * stride;
        h[r] = uH[i < n ? i : (uint64_t)n - 1];
    }

    uint32_t want_hi = 0;
    if (PASS > 0) {
        if (tid < 64) {
            uint32_t bin, rem;
            if (PASS == 1) pick_bin<kDigit0Bins>(hist0 + (uint64_t)u * kDigit0Bins, k, &bin, &rem);
            else pick_bin_two_level(ucoarse, upartial, hb, ust[ST_KREM0], &bin, &rem);
            if (lane == 0) {
                chosen[0] = bin;
                chosen[1] = rem;
                if (blockIdx.x == 0) { ust[ST_BIN0 + PASS - 1] = bin; ust[ST_KREM0 + PASS - 1] = rem; }
            }
        }
        __syncthreads();
        want_hi = PASS == 1 ? chosen[0] : ((ust[ST_BIN0] << 11) | chosen[0]);
    } else {
        __syncthreads();
    }

    constexpr int shift = PASS == 0 ? 22 : (PASS == 1 ? 11 : 0);
    constexpr uint32_t mask = PASS == 0 ? 1023u : 2047u;
    constexpr int hi_shift = PASS == 1 ? 22 : 11;

    for (uint64_t base = base0; base < n; base += R * stride) {
        uint32_t key[R];
        bool ok[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            ok[r] = base + r * stride < n;
            key[r] = order_key(h[r]);
        }
        // the next sixteen, while these are counted
        if (base + R * stride < n) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint64_t i = base + (R + r) * stride;
                h[r] = uH[i < n ? i : (uint64_t)n - 1];
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            bool active = ok[r] && (PASS == 0 || (key[r] >> hi_shift) == want_hi);
            const uint32_t bin = (key[r] >> shift) & mask;
#pragma unroll 1
            for (int it = 0; it < PEEL; ++it) {
                const uint64_t am = __ballot(active);
                if (am == 0) break;
                const int leader = (int)__ffsll((unsigned long long)am) - 1;
                const uint32_t lb = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
                const bool same = active && bin == lb;
                const uint64_t sm = __ballot(same);
                if (lane == leader) atomicAdd(&lh[lb], (uint32_t)__popcll(sm));
                active = active && !same;
            }
            if (active) atomicAdd(&lh[bin], 1u);
        }
    }
    __syncthreads();
    if (PASS == 0) {
        for (int i = tid; i < BINS; i += 256)
            if (lh[i]) atomicAdd(&hist0[(uint64_t)u * kDigit0Bins + i], lh[i]);
    } else {
        // my histogram with plain stores; only the 64 super-bin totals go through atomics
        uint32_t *mine = upartial + ((uint64_t)(PASS - 1) * hb + blockIdx.x) * kHistBins;
        for (int i = tid; i < BINS; i += 256) mine[i] = lh[i];
        if (tid < 64) {
            uint32_t tot = 0;
#pragma unroll 8
            for (int i = 0; i < 32; ++i) tot += lh[32 * tid + ((i + tid) & 31)];     // rotated: no bank conflicts
            if (tot) atomicAdd(&ucoarse[(PASS - 1) * 64 + tid], tot);
        }
    }
}

// Per segment of kSegTiles tiles (one wavefront each): how many keys equal K* and how many exceed it.
// K* and `take` come from the pass-2 histogram; every block derives them, block 0 records them.
__global__ __launch_bounds__(256) void k_seg_count(const float *__restrict__ H, uint32_t n, uint32_t nseg,
                                                   const uint32_t *__restrict__ coarse,
                                                   const uint32_t *__restrict__ partial, uint32_t hb,
                                                   uint32_t *__restrict__ state, uint32_t *__restrict__ seg)
{
    __shared__ uint32_t chosen[2];
    const uint32_t u = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t *ust = state + (uint64_t)u * 8;
    // my wavefront's segment: its sixteen keys per lane are requested first (clamped index, nothing behind a
    // branch); the threshold they are compared with is worked out while they arrive
    constexpr int KEYS = (int)(kSegTiles / 64);
    const uint32_t s = blockIdx.x * 4 + wave;
    const float *uH = H + (uint64_t)u * n;
    float h[KEYS];
#pragma unroll
    for (int r = 0; r < KEYS; ++r) {
        const uint64_t j = (uint64_t)s * kSegTiles + (uint64_t)r * 64 + lane;
        h[r] = uH[j < n ? j : (uint64_t)n - 1];
    }
    if (tid < 64) {
        uint32_t bin, rem;
        pick_bin_two_level(coarse + ((uint64_t)u * 2 + 1) * 64, partial + ((uint64_t)u * 2 + 1) * hb * kHistBins, hb,
                           ust[ST_KREM1], &bin, &rem);
        const uint32_t key = (ust[ST_BIN0] << 22) | (ust[ST_BIN1] << 11) | bin;
        if (lane == 0) {
            chosen[0] = key;
            chosen[1] = rem;
            if (blockIdx.x == 0) { ust[ST_BIN2] = bin; ust[ST_KEY] = key; ust[ST_TAKE] = rem; }
        }
    }
    __syncthreads();
    const uint32_t thr = chosen[0];
    if (s >= nseg) return;
    uint32_t eq = 0, gt = 0;
#pragma unroll
    for (int r = 0; r < KEYS; ++r) {
        const bool ok = (uint64_t)s * kSegTiles + (uint64_t)r * 64 + lane < n;
        const uint32_t key = order_key(h[r]);
        eq += (uint32_t)__popcll(__ballot(ok && key == thr));
        gt += (uint32_t)__popcll(__ballot(ok && key > thr));
    }
    if (lane == 0) {
        seg[((uint64_t)u * nseg + s) * 2 + 0] = eq;
        seg[((uint64_t)u * nseg + s) * 2 + 1] = gt;
    }
}

// Width bit of every tile, rank-table entries, and the bit map itself when units start on 64-tile
// boundaries (otherwise one byte per tile goes to `sel_bytes` and k_bitmap_pack follows).
// A block owns 4 consecutive segments.  Its first wavefront sums the segment counts that precede
// the block: equal keys before it (they are taken in index order until `take` are used up) and
// wide tiles before it (every earlier ranking unit contributes exactly k).
__global__ __launch_bounds__(256) void k_assign(const float *__restrict__ H, uint32_t n, uint32_t k, uint32_t nseg,
                                                const uint32_t *__restrict__ state,
                                                const uint32_t *__restrict__ seg,
                                                uint64_t *__restrict__ bitmap, uint32_t *__restrict__ ranks,
                                                uint8_t *__restrict__ sel_bytes, int aligned)
{
    __shared__ uint32_t base_eq[4], base_rank[4];
    const uint32_t u = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t *ust = state + (uint64_t)u * 8;
    const uint32_t thr = ust[ST_KEY], take = ust[ST_TAKE];
    const uint32_t *useg = seg + (uint64_t)u * nseg * 2;
    const uint32_t s0 = blockIdx.x * 4;
    // my wavefront's segment: its sixteen keys per lane are requested first (clamped index, nothing behind a
    // branch) and arrive while the first wavefront sums the counts of the segments before this block
    constexpr int KEYS = (int)(kSegTiles / 64);
    const float *uH = H + (uint64_t)u * n;
    float h[KEYS];
#pragma unroll
    for (int r = 0; r < KEYS; ++r) {
        const uint64_t jl = (uint64_t)(s0 + wave) * kSegTiles + (uint64_t)r * 64 + lane;
        h[r] = uH[jl < n ? jl : (uint64_t)n - 1];
    }

    if (tid < 64) {
        // Sums over the s0 segments before this block, 512 segments per sweep: lane l owns the 8 consecutive
        // segments 8l .. 8l+7 of the sweep (loaded at once), a wave scan orders the lanes, `eq_run` / `rank_run`
        // carry the totals from sweep to sweep.
        const uint2 *pairs = reinterpret_cast<const uint2 *>(useg);
        uint32_t eq_run = 0, rank_run = u * k;
        for (uint32_t base = 0; base < s0; base += 512) {
            uint2 e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t sidx = base + (uint32_t)lane * 8 + i;
                e[i] = pairs[sidx < s0 ? sidx : 0u];                 // clamped, not branched; masked below
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (base + (uint32_t)lane * 8 + i >= s0) e[i] = make_uint2(0u, 0u);
            uint32_t eq_sum = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) eq_sum += e[i].x;
            const uint32_t eq_incl = wave_incl_scan(eq_sum);
            uint32_t eq_before = eq_run + eq_incl - eq_sum;
            uint32_t sel_sum = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t left = eq_before < take ? take - eq_before : 0u;
                sel_sum += e[i].y + (e[i].x < left ? e[i].x : left);
                eq_before += e[i].x;
            }
            const uint32_t sel_incl = wave_incl_scan(sel_sum);
            eq_run += (uint32_t)__shfl((int)eq_incl, 63, 64);
            rank_run += (uint32_t)__shfl((int)sel_incl, 63, 64);
        }
        // the block's own four segments, in order
        uint2 own[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) own[w] = pairs[s0 + w < nseg ? s0 + w : nseg - 1];
#pragma unroll
        for (int w = 0; w < 4; ++w)
            if (s0 + w >= nseg) own[w] = make_uint2(0u, 0u);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (lane == 0) { base_eq[w] = eq_run; base_rank[w] = rank_run; }
            const uint32_t left = eq_run < take ? take - eq_run : 0u;
            rank_run += own[w].y + (own[w].x < left ? own[w].x : left);
            eq_run += own[w].x;
        }
    }
    __syncthreads();
    const uint32_t s = s0 + wave;
    if (s >= nseg) return;
    uint32_t eq_run = base_eq[wave], rank_run = base_rank[wave];
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < KEYS; ++r) {
        const uint64_t jl = (uint64_t)s * kSegTiles + (uint64_t)r * 64 + lane;
        const bool ok = jl < n;
        const uint32_t key = order_key(h[r]);
        const bool eq = ok && key == thr;
        const uint64_t eq_mask = __ballot(eq);
        const bool sel = ok && (key > thr || (eq && eq_run + (uint32_t)__popcll(eq_mask & below) < take));
        const uint64_t sel_mask = __ballot(sel);
        const uint64_t jg = (uint64_t)u * n + jl;     // tile index in the tensor
        if (aligned) {
            if (lane == 0 && ok) { bitmap[jg >> 6] = sel_mask; ranks[jg >> 6] = rank_run; }
        } else if (ok) {
            sel_bytes[jg] = sel ? 1 : 0;
            if ((jg & 63u) == 0) ranks[jg >> 6] = rank_run + (uint32_t)__popcll(sel_mask & below);
        }
        eq_run += (uint32_t)__popcll(eq_mask);
        rank_run += (uint32_t)__popcll(sel_mask);
    }
}

__global__ __launch_bounds__(256) void k_bitmap_pack(const uint8_t *__restrict__ sel_bytes, uint32_t T,
                                                     uint64_t *__restrict__ bitmap)
{
    const uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t word = __ballot(j < T && sel_bytes[j < T ? j : 0] != 0);
    if ((threadIdx.x & 63) == 0 && (j >> 6) < ((uint64_t)T + 63) / 64) bitmap[j >> 6] = word;
}

// Allocation tiles of m > 1 quantization tiles (Sec. 3.2): the selection ran over allocation tiles and left
// one byte per allocation tile in `sel_a` and, in `ranks_a`, the wide allocation tiles before each group of
// 64.  This kernel writes the stream's bit map and rank table over QUANTIZATION tiles: tile j takes the
// width of allocation tile j / m, and the wide quantization tiles before j are m times the wide
// allocation tiles before j / m, plus j % m if its own allocation tile is wide.  One wavefront per
// 64 quantization tiles.
__global__ __launch_bounds__(256) void k_expand_alloc(const uint8_t *__restrict__ sel_a,
                                                      const uint32_t *__restrict__ ranks_a, uint32_t T, uint32_t m,
                                                      uint64_t *__restrict__ bitmap, uint32_t *__restrict__ ranks)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t j0 = j - lane;
    if (j0 >= T) return;                               // whole wavefront past the end
    const uint32_t ja0 = j0 / m, r0 = j0 % m;
    const uint32_t base = ja0 & ~63u;
    const bool before = base + lane < ja0 && sel_a[base + lane] != 0;
    const uint32_t rank_a = ranks_a[ja0 >> 6] + (uint32_t)__popcll(__ballot(before));
    const bool mine = j < T && sel_a[j < T ? j / m : 0] != 0;
    const uint64_t word = __ballot(mine);
    if (lane == 0) {
        bitmap[j0 >> 6] = word;
        ranks[j0 >> 6] = rank_a * m + (sel_a[ja0] != 0 ? r0 : 0u);
    }
}

constexpr uint32_t kBlockSelectThreads = 1024;

// LDS scratch of block_radix_select.
struct BlockSelectLds {
    uint32_t copies[8192];                       // the histogram of one digit, several copies of every bin
    uint32_t lh[4096 + 64];                      // its bins added up; bin b at b + b/64: a lane that reads bin l of a chunk
                                                 // of 64 bins while its neighbours read theirs meets no bank conflict
    uint32_t chunk_total[64];                    // totals of the chunks of 64 bins
    uint32_t chosen[5];                          // bin, wanted inside it, its count; smallest and largest value
};

// Run by the first wavefront: the bin of L.lh that holds the `want`-th largest value, in two levels -- the chunk of 64
// bins from the top (totals in L.chunk_total; chunks that are not in use hold 0), then the bin inside it.  Leaves the
// bin, the number still wanted inside it and its count in L.chosen[0..2].
__device__ __forceinline__ void pick_from_chunks(BlockSelectLds &L, uint32_t want, int lane)
{
    const uint32_t cs = L.chunk_total[63 - lane];                           // lane l: chunk 63 - l, from the top
    const uint32_t above = wave_incl_scan(cs) - cs;
    const uint64_t who = __ballot(above < want && want <= above + cs);
    const int src = who ? (int)__ffsll((unsigned long long)who) - 1 : 0;
    const uint32_t chunk = 63u - (uint32_t)src;
    const uint32_t want2 = want - (uint32_t)__shfl((int)above, src, 64);
    const uint32_t bs = L.lh[chunk * 65 + (63 - lane)];                     // lane l: bin 63 - l of the chunk
    const uint32_t above2 = wave_incl_scan(bs) - bs;
    const uint64_t who2 = __ballot(above2 < want2 && want2 <= above2 + bs);
    const int src2 = who2 ? (int)__ffsll((unsigned long long)who2) - 1 : 0;
    if (lane == src2) {
        L.chosen[0] = chunk * 64 + (63u - (uint32_t)src2);
        L.chosen[1] = want2 - above2;
        L.chosen[2] = bs;
    }
}

// Workgroup-wide radix select over the values that `each` hands to its argument (every thread visits its own share
// of the values; each(g) calls g(value) for each of them): the `want`-th largest value (1 <= want <= number of values),
// how many values equal to it belong to the `want` largest, and how many values equal to it there are.  The values of
// one selection lie close together (the entropies of one sample, or the keys of one histogram bin), so the digits are
// taken from value - minimum: 12 bits at a time from the top of max - min, usually two passes.  Called by all 1024
// threads; the result is the same in every thread.
template <class Each>
__device__ __forceinline__ void block_radix_select(uint32_t want, Each each, BlockSelectLds &L, uint32_t *thr_out,
                                                   uint32_t *take_out, uint32_t *equal_out)
{
    constexpr int kBins = 4096;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid == 0) { L.chosen[3] = 0xffffffffu; L.chosen[4] = 0u; }
    __syncthreads();
    {
        uint32_t lo = 0xffffffffu, hi = 0u;
        each([&](uint32_t val) { lo = val < lo ? val : lo; hi = val > hi ? val : hi; });
        // per wavefront first: a thousand atomics on one LDS address would take longer than the rest of the selection
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint32_t olo = (uint32_t)__shfl_xor((int)lo, off, 64), ohi = (uint32_t)__shfl_xor((int)hi, off, 64);
            lo = olo < lo ? olo : lo;
            hi = ohi > hi ? ohi : hi;
        }
        if (lane == 0 && lo <= hi) { atomicMin(&L.chosen[3], lo); atomicMax(&L.chosen[4], hi); }
    }
    __syncthreads();
    const uint32_t vmin = L.chosen[3], span = L.chosen[4] - vmin;
    int bits = 32 - __builtin_clz(span | 1u);    // digits cover bits [0, bits) of value - vmin
    uint32_t prefix = 0;                         // the digits found so far, as the top bits of value - vmin
    uint32_t equal = 0;
#pragma unroll 1
    while (true) {
        const int shift = bits > 12 ? bits - 12 : 0;         // this pass: bits [shift, bits)
        const uint32_t mask = (1u << (bits - shift)) - 1u;
        // Several copies of every bin, indexed by the lane, as many as the 8192 words hold (2 for a 12-bit digit, at
        // most 32): a wavefront's atomics on one LDS address are serialized, and under massive ties a digit takes
        // one or two values.
        const int copy_bits = 13 - (bits - shift) > 5 ? 5 : 13 - (bits - shift);
        const uint32_t my_copy = (uint32_t)lane & ((1u << copy_bits) - 1u);
#pragma unroll
        for (int i = 0; i < 8; ++i) L.copies[i * (int)kBlockSelectThreads + tid] = 0;
        __syncthreads();
        each([&](uint32_t val) {
            const uint32_t d = val - vmin;
            if (bits == 32 || (d >> bits) == prefix) atomicAdd(&L.copies[(((d >> shift) & mask) << copy_bits) | my_copy], 1u);
        });
        __syncthreads();
        // thread t adds up the copies of bins t, t + 1024, ...; the 64 bins of a wavefront are one chunk, whose total
        // the wavefront leaves beside them
#pragma unroll
        for (int part = 0; part < kBins / (int)kBlockSelectThreads; ++part) {
            const uint32_t bin = (uint32_t)tid + kBlockSelectThreads * part;
            uint32_t sum = 0;
            if (bin <= mask) {
                for (int c = 0; c < (1 << copy_bits); ++c) sum += L.copies[(bin << copy_bits) + c];
            }
            L.lh[bin + (bin >> 6)] = sum;
            const uint32_t upto = wave_incl_scan(sum);
            if (lane == 63) L.chunk_total[(kBlockSelectThreads / 64) * part + wave] = upto;
        }
        __syncthreads();
        if (tid < 64) pick_from_chunks(L, want, lane);
        __syncthreads();
        prefix = (bits - shift == 32) ? L.chosen[0] : ((prefix << (bits - shift)) | L.chosen[0]);
        want = L.chosen[1];
        equal = L.chosen[2];
        __syncthreads();
        if (shift == 0) break;
        bits = shift;
    }
    *thr_out = vmin + prefix;
    *take_out = want;
    *equal_out = equal;
}

// ---- small ranking units: the whole selection in one launch

constexpr uint32_t kSmallUnitThreads = kBlockSelectThreads;
#ifndef TAHQ_SMALL_UNIT_MAX
#define TAHQ_SMALL_UNIT_MAX 32768
#endif
constexpr uint32_t kSmallUnitMaxKeys = TAHQ_SMALL_UNIT_MAX;    // 32 keys per thread; beyond that the keys no longer fit the
                                                 // register file of a 1024-thread workgroup and the multi-launch path is as fast

// A ranking unit of at most 1024 * KPT keys, ranked by ONE workgroup that keeps the keys in registers: the
// radix passes (12 bits at a time of key - smallest key, two passes as a rule) run on an LDS histogram, the per-group counts and their prefix sums stay in LDS, and
// the bit map and rank table (or, for units that do not start on 64-tile boundaries, one byte per tile and
// the rank entries of the 64-tile groups) are written at the end.  Same result as k_radix_pass x 3,
// k_seg_count and k_assign, in one launch instead of five: small tensors are bound by launch latency.
// Wavefront w owns the KPT consecutive 64-tile groups KPT*w ..: thread (w, lane l) holds, for r = 0 .. KPT-1, the
// key of tile 64 * (KPT w + r) + l of the unit.  KPT is 16 or 32.
template <int KPT>
__global__ __launch_bounds__(kSmallUnitThreads) void k_select_small(const float *__restrict__ H, uint32_t n, uint32_t k,
                                                                    uint64_t *__restrict__ bitmap,
                                                                    uint32_t *__restrict__ ranks,
                                                                    uint8_t *__restrict__ sel_bytes, int aligned)
{
    constexpr int NG = 16 * KPT;                 // 64-tile groups the workgroup can hold
    constexpr int PER = NG / 64;                 // lane l of wavefront 0 scans the PER consecutive groups PER*l ..
    __shared__ BlockSelectLds L;
    __shared__ uint32_t grp_eq[NG], grp_sel[NG];
    const uint32_t u = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *uH = H + (uint64_t)u * n;
    const uint64_t below = (1ull << lane) - 1ull;

    // all loads first (from a clamped index, so that none of them sits behind a branch), then the keys
    float h[KPT];
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
        const uint32_t i = (uint32_t)(KPT * wave + r) * 64u + lane;
        h[r] = uH[i < n ? i : n - 1];
    }
    uint32_t key[KPT];
#pragma unroll
    for (int r = 0; r < KPT; ++r) key[r] = order_key(h[r]);
    auto in_unit = [&](int r) { return (uint32_t)(KPT * wave + r) * 64u + lane < n; };

    // the k-th largest key, how many tiles equal to it are taken, and how many there are
    uint32_t thr, take, equal;
    block_radix_select(k, [&](auto &&visit) {
#pragma unroll
        for (int r = 0; r < KPT; ++r) {
            if (in_unit(r)) visit(key[r]);
        }
    }, L, &thr, &take, &equal);

    // The width bit of every tile; lane r keeps the bit map word of the wavefront's r-th group.
    uint64_t my_word = 0;
    if (take == equal) {
        // every tile whose key equals the threshold is taken (one such tile, as a rule)
#pragma unroll
        for (int r = 0; r < KPT; ++r) {
            const bool sel = in_unit(r) && key[r] >= thr;
            const uint64_t selm = __ballot(sel);
            if (lane == r) my_word = selm;
            if (!aligned && in_unit(r)) sel_bytes[(uint64_t)u * n + (uint64_t)(KPT * wave + r) * 64u + lane] = sel ? 1 : 0;
        }
    } else {
        // Keys equal to thr are taken in index order until `take` are used up, so every group needs the number of
        // equal keys before it: lane r keeps the count of the wavefront's r-th group, wavefront 0 scans the groups.
        uint32_t my_eq = 0;
#pragma unroll
        for (int r = 0; r < KPT; ++r) {
            const uint32_t ne = (uint32_t)__popcll(__ballot(in_unit(r) && key[r] == thr));
            if (lane == r) my_eq = ne;
        }
        if (lane < KPT) grp_eq[KPT * wave + lane] = my_eq;
        __syncthreads();
        if (tid < 64) {
            uint32_t e[PER], esum = 0;
#pragma unroll
            for (int i = 0; i < PER; ++i) { e[i] = grp_eq[lane * PER + i]; esum += e[i]; }
            uint32_t eq_before = wave_incl_scan(esum) - esum;
#pragma unroll
            for (int i = 0; i < PER; ++i) { grp_eq[lane * PER + i] = eq_before; eq_before += e[i]; }
        }
        __syncthreads();
        const uint32_t my_eq_before = lane < KPT ? grp_eq[KPT * wave + lane] : 0u;
#pragma unroll
        for (int r = 0; r < KPT; ++r) {
            const bool ok = in_unit(r);
            const bool eq = ok && key[r] == thr;
            const uint64_t eqm = __ballot(eq);
            bool sel = ok && key[r] > thr;
            if (eqm) {                           // at most a few groups hold keys equal to the threshold, as a rule
                const uint32_t eq_before = (uint32_t)__builtin_amdgcn_readlane((int)my_eq_before, r);
                sel = sel || (eq && eq_before + (uint32_t)__popcll(eqm & below) < take);
            }
            const uint64_t selm = __ballot(sel);
            if (lane == r) my_word = selm;
            if (!aligned && ok) sel_bytes[(uint64_t)u * n + (uint64_t)(KPT * wave + r) * 64u + lane] = sel ? 1 : 0;
        }
    }
    if (lane < KPT) grp_sel[KPT * wave + lane] = (uint32_t)__popcll(my_word);
    __syncthreads();
    if (tid < 64) {
        uint32_t c[PER], csum = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) { c[i] = grp_sel[lane * PER + i]; csum += c[i]; }
        uint32_t rank_before = wave_incl_scan(csum) - csum;
#pragma unroll
        for (int i = 0; i < PER; ++i) { grp_sel[lane * PER + i] = rank_before; rank_before += c[i]; }
    }
    __syncthreads();
    // lane r writes what belongs to the wavefront's r-th group
    const uint32_t g = (uint32_t)(KPT * wave + lane);
    if (lane < KPT && g * 64u < n) {
        const uint32_t rank = u * k + grp_sel[g];            // wide tiles before the group, in the whole tensor
        const uint64_t j0 = (uint64_t)u * n + (uint64_t)g * 64u;     // the group's first tile in the tensor
        if (aligned) {
            bitmap[j0 >> 6] = my_word;
            ranks[j0 >> 6] = rank;
        } else {
            // units do not start on 64-tile boundaries: the rank-table entry of the boundary inside this group
            // (if the group still reaches it)
            const uint32_t p = (uint32_t)((64u - (uint32_t)(j0 & 63u)) & 63u);        // distance to the boundary
            if (g * 64u + p < n) ranks[(j0 + p) >> 6] = rank + (uint32_t)__popcll(my_word & ((1ull << p) - 1ull));
        }
    }
}

// ---- large ranking units: the selection in two launches after the entropy kernel
//
// The entropy kernel leaves, per ranking unit, a histogram of the entropies over kLinBins linear bins.  The bin of an
// entropy is non-decreasing in it, so the k-th largest entropy lies in the bin b* where the counts, summed from the
// top, reach k: every tile in a higher bin is selected, every tile in a lower bin is not, and only the tiles IN
// bin b* (about one in a few hundred for activations) need an exact ranking for the `rem` places that are left.
//
//   k_select_classify (workgroups of 1024 threads over blocks of 16384 tiles): find b*; write the bit map words with
//     the tiles above b* and the block's count of them; append (key, tile) of the tiles in b* to the unit's
//     candidate list.
//   k_select_resolve (same grid): every workgroup ranks the unit's candidates exactly for itself -- radix select on
//     the keys, then, among the keys equal to the threshold, by tile index, so that ties go to the lower index
//     whatever order the list came in -- adds the selected candidates of its own block to the block's bit map
//     words, and writes the block's part of the rank table (tiles above b* in the blocks before it, from the
//     counts; selected candidates before it, counted while ranking).  Ranking a few thousand candidates sixteen to
//     thirty-two times over costs less than one workgroup walking the unit's whole bit map.
// If a unit's bin b* holds more tiles than the list does (massive ties), the unit's first workgroup of the second
// kernel does all of it alone, straight from the entropies: slower but as exact.  Needs ranking units that start on
// 64-tile boundaries.
// (One launch, with the last workgroup of every unit doing the second part, measured ten times slower: what a
// workgroup wrote becomes visible to a workgroup on another XCD only through fences that write back the L2.)

constexpr uint32_t kFusedThreads = kBlockSelectThreads;
constexpr uint32_t kFusedKeysPerBlock = 16 * kFusedThreads;

__global__ __launch_bounds__(kFusedThreads) void k_select_classify(const float *__restrict__ H, uint32_t n, uint32_t k,
                                                                   float bin_scale,
                                                                   const uint32_t *__restrict__ lin_hist,
                                                                   uint32_t *__restrict__ fused,
                                                                   uint2 *__restrict__ cand,
                                                                   uint32_t *__restrict__ block_above,
                                                                   uint64_t *__restrict__ bitmap)
{
    constexpr int KPT = 16;                      // keys per thread: wavefront w owns 16 groups of 64 tiles
    __shared__ uint32_t chosen[2];
    __shared__ uint32_t wave_cand[kFusedThreads / 64], wave_above[kFusedThreads / 64];
    const uint32_t u = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const float *uH = H + (uint64_t)u * n;
    uint32_t *listed = fused + (uint64_t)u * 4;              // candidates listed so far
    uint2 *ucand = cand + (uint64_t)u * kCandCap;
    uint64_t *ubitmap = bitmap + (((uint64_t)u * n) >> 6);   // units start on 64-tile boundaries
    const uint32_t ngroups = n >> 6;

    // all loads first (from a clamped index: none of them sits behind a branch)
    const uint32_t group0 = blockIdx.x * (kFusedKeysPerBlock / 64) + (uint32_t)(KPT * wave);
    float h[KPT];
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
        const uint32_t i = (group0 + r) * 64u + lane;
        h[r] = uH[i < n ? i : n - 1];
    }
    if (tid < 64) {
        uint32_t bin, rem;
        pick_bin<kLinBins>(lin_hist + (uint64_t)u * kLinBins, k, &bin, &rem);
        if (lane == 0) { chosen[0] = bin; chosen[1] = rem; }
    }
    __syncthreads();
    const uint32_t bstar = chosen[0];

    uint32_t bins[KPT];
    uint64_t my_word = 0;
    uint32_t n_cand = 0, n_above = 0;            // of my wavefront (the same in every lane)
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
        const bool ok = (group0 + r) * 64u + lane < n;
        bins[r] = ok ? linear_bin(h[r], bin_scale) : 0xffffffffu;
        const uint64_t above = __ballot(ok && bins[r] > bstar);
        if (lane == r) my_word = above;
        n_above += (uint32_t)__popcll(above);
        n_cand += (uint32_t)__popcll(__ballot(bins[r] == bstar));
    }
    if (lane < KPT && group0 + lane < ngroups) ubitmap[group0 + lane] = my_word;
    // one place in the list for the whole workgroup (a unit's workgroups all add to one counter: few, large additions)
    if (lane == 0) { wave_cand[wave] = n_cand; wave_above[wave] = n_above; }
    __syncthreads();
    if (tid == 0) {
        uint32_t total = 0, above = 0;
        for (int w = 0; w < (int)(kFusedThreads / 64); ++w) { total += wave_cand[w]; above += wave_above[w]; }
        chosen[1] = total ? atomicAdd(listed, total) : 0u;
        block_above[(uint64_t)u * gridDim.x + blockIdx.x] = above;
    }
    __syncthreads();
    if (n_cand != 0) {
        uint32_t base = chosen[1];
        for (int w = 0; w < wave; ++w) base += wave_cand[w];
        base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
#pragma unroll
        for (int r = 0; r < KPT; ++r) {
            const uint64_t m = __ballot(bins[r] == bstar);
            if (bins[r] == bstar) {
                const uint32_t pos = base + bits_below_me(m);
                if (pos < kCandCap) ucand[pos] = make_uint2(order_key(h[r]), (group0 + r) * 64u + lane);
            }
            base += (uint32_t)__popcll(m);
        }
    }
}

// LDS of k_select_resolve
struct ResolveLds {
    BlockSelectLds sel;
    uint32_t chosen[4];                          // threshold bin, wanted inside it; threshold sub-bin, wanted inside it
    uint32_t n_equal, n_before;
    uint32_t equal_tile[kFusedThreads];          // tiles whose key equals the threshold (the first 1024)
    uint32_t wave_total[kFusedThreads / 64];
    uint32_t words[2 * (kFusedKeysPerBlock / 64)];           // the block's bit map words, as dwords
};

// Which of the candidates f visits are selected: `rem` of them, by (key descending, tile ascending).  each_candidate(f)
// calls f(key, tile) for my share of the tiles in bin b*; take_it(tile) is called for every selected one.  All 1024
// threads.
template <class EachCandidate, class TakeIt>
__device__ __forceinline__ void rank_candidates(uint32_t rem, EachCandidate each_candidate, TakeIt take_it, ResolveLds &L)
{
    const int tid = threadIdx.x;
    if (tid == 0) L.n_equal = 0;
    uint32_t thr, take, equal;
    block_radix_select(rem, [&](auto g) { each_candidate([&](uint32_t key, uint32_t) { g(key); }); }, L.sel, &thr, &take,
                       &equal);
    if (take == equal) {                         // every tile equal to the threshold is taken (one, as a rule)
        each_candidate([&](uint32_t key, uint32_t tile) { if (key >= thr) take_it(tile); });
        return;
    }
    // tiles above the threshold are taken; of those equal to it, the `take` with the lowest tile indices
    each_candidate([&](uint32_t key, uint32_t tile) {
        if (key > thr) take_it(tile);
        else if (key == thr) {
            const uint32_t at = atomicAdd(&L.n_equal, 1u);
            if (at < kFusedThreads) L.equal_tile[at] = tile;
        }
    });
    __syncthreads();
    const uint32_t ne = L.n_equal;
    if (ne <= kFusedThreads) {
        // a handful, as a rule: thread t ranks the t-th of them among all of them
        if ((uint32_t)tid < ne) {
            const uint32_t mine = L.equal_tile[tid];
            uint32_t lower = 0;
            for (uint32_t i = 0; i < ne; ++i) lower += L.equal_tile[i] < mine ? 1u : 0u;
            if (lower < take) take_it(mine);
        }
    } else {
        uint32_t thr_index, unused, unused2;     // a tile with key == thr is taken iff ~tile >= thr_index
        block_radix_select(take, [&](auto g) {
            each_candidate([&](uint32_t key, uint32_t tile) { if (key == thr) g(~tile); });
        }, L.sel, &thr_index, &unused, &unused2);
        each_candidate([&](uint32_t key, uint32_t tile) { if (key == thr && ~tile >= thr_index) take_it(tile); });
    }
}

// The overflow path: one workgroup resolves a whole unit from the entropies (bin b* holds more tiles than the list).
__device__ __noinline__ void resolve_unit_alone(const float *__restrict__ uH, uint32_t n, uint32_t rank_base,
                                                float bin_scale, uint32_t bstar, uint32_t rem,
                                                uint64_t *__restrict__ ubitmap, uint32_t *__restrict__ uranks,
                                                ResolveLds &L)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t ngroups = n >> 6;
    uint32_t *ubits32 = reinterpret_cast<uint32_t *>(ubitmap);
    if (rem != 0) {
        rank_candidates(rem, [&](auto f) {
            for (uint32_t i = tid; i < n; i += kFusedThreads) {
                const float hv = uH[i];
                if (linear_bin(hv, bin_scale) == bstar) f(order_key(hv), i);
            }
        }, [&](uint32_t tile) { atomicOr(&ubits32[tile >> 5], 1u << (tile & 31u)); }, L);
    }
    // every wavefront's atomics have been performed (acknowledged by the L2, where the loads below read) before
    // anybody reads the words
    __builtin_amdgcn_s_waitcnt(0x0f70);          // vmcnt(0)
    __syncthreads();
    // the unit's rank table from the finished bit map (read where the atomics were performed, in the L2: this
    // workgroup's L1 may hold older copies of some words); a thread takes eight consecutive groups per sweep
    constexpr int GPT = 8;
    uint32_t running = rank_base;
    for (uint32_t g0 = 0; g0 < ngroups; g0 += GPT * kFusedThreads) {
        const uint32_t first = g0 + (uint32_t)tid * GPT;
        uint32_t c[GPT], mine = 0;
#pragma unroll
        for (int i = 0; i < GPT; ++i) {
            const uint32_t g = first + i < ngroups ? first + i : ngroups - 1;      // clamped, masked below
            const uint32_t lo = __hip_atomic_load(&ubits32[2 * g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t hi = __hip_atomic_load(&ubits32[2 * g + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c[i] = first + i < ngroups ? (uint32_t)__popc(lo) + (uint32_t)__popc(hi) : 0u;
            mine += c[i];
        }
        const uint32_t incl = wave_incl_scan(mine);
        if (lane == 63) L.wave_total[wave] = incl;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < (int)(kFusedThreads / 64); ++w) {
            const uint32_t wt = L.wave_total[w];
            if (w < wave) before += wt;
            total += wt;
        }
        uint32_t rank = running + before + incl - mine;
#pragma unroll
        for (int i = 0; i < GPT; ++i) {
            if (first + i < ngroups) uranks[first + i] = rank;
            rank += c[i];
        }
        running += total;
        __syncthreads();
    }
}

__global__ __launch_bounds__(kFusedThreads) void k_select_resolve(const float *__restrict__ H, uint32_t n, uint32_t k,
                                                                  float bin_scale,
                                                                  const uint32_t *__restrict__ lin_hist,
                                                                  const uint32_t *__restrict__ fused,
                                                                  const uint2 *__restrict__ cand,
                                                                  const uint32_t *__restrict__ block_above,
                                                                  uint64_t *__restrict__ bitmap,
                                                                  uint32_t *__restrict__ ranks)
{
    __shared__ ResolveLds L;
    constexpr uint32_t GROUPS = kFusedKeysPerBlock / 64;     // 64-tile groups of a block
    const uint32_t u = blockIdx.y, blk = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const float *uH = H + (uint64_t)u * n;
    const uint2 *ucand = cand + (uint64_t)u * kCandCap;
    uint64_t *ubitmap = bitmap + (((uint64_t)u * n) >> 6);
    uint32_t *uranks = ranks + (((uint64_t)u * n) >> 6);
    const uint32_t ngroups = n >> 6;
    const uint32_t group0 = blk * GROUPS;
    const uint32_t mygroups = ngroups - group0 < GROUPS ? ngroups - group0 : GROUPS;

    // everything this workgroup reads from global memory, requested at once: the candidates (sixteen per thread; the
    // list always has room for them, what lies beyond its end is ignored), the block's words, the counts of the
    // blocks before it, the histogram
    constexpr int CPT = (int)(kCandCap / kFusedThreads);
    uint2 c[CPT];
#pragma unroll
    for (int r = 0; r < CPT; ++r) c[r] = ucand[(uint32_t)r * kFusedThreads + tid];
    const uint32_t listed = fused[(uint64_t)u * 4];
    uint64_t my_word = 0;
    if ((uint32_t)tid < mygroups) my_word = ubitmap[group0 + tid];
    uint32_t above_before = 0;
    for (uint32_t b = tid; b < blk; b += kFusedThreads) above_before += block_above[(uint64_t)u * gridDim.x + b];
    if (tid < 64) {
        uint32_t bin, rem;
        pick_bin<kLinBins>(lin_hist + (uint64_t)u * kLinBins, k, &bin, &rem);
        if (lane == 0) { L.chosen[0] = bin; L.chosen[1] = rem; }
    }
    if (tid == 0) { L.n_before = 0; L.n_equal = 0; }
    static_assert(kSubBins == kFusedThreads, "one sub-bin per thread");
    uint32_t *sub_hist = L.sel.copies;           // the threshold bin's candidates by sub-bin
    sub_hist[tid] = 0;
    if ((uint32_t)tid < GROUPS) { L.words[2 * tid] = (uint32_t)my_word; L.words[2 * tid + 1] = (uint32_t)(my_word >> 32); }
    __syncthreads();
    const uint32_t bstar = L.chosen[0], rem = L.chosen[1];
    __syncthreads();                             // `chosen` is used again below

    if (listed > kCandCap) {
        if (blk == 0) resolve_unit_alone(uH, n, u * k, bin_scale, bstar, rem, ubitmap, uranks, L);
        return;
    }
    // the selected candidates: those of my block go into its words, those before it are counted
    const uint32_t first_tile = group0 * 64u;
    uint32_t before = 0;
    auto take_it = [&](uint32_t tile) {
        if (tile < first_tile) ++before;
        else if (tile - first_tile < kFusedKeysPerBlock) atomicOr(&L.words[(tile - first_tile) >> 5], 1u << (tile & 31u));
    };
    if (rem != 0) {
        // A histogram of the candidates over 1024 sub-bins of their bin narrows the threshold down once more:
        // candidates in a higher sub-bin are selected, those in the threshold's own sub-bin (a handful, as a rule) are
        // ranked directly, thread t placing the t-th of them among all of them by (key descending, tile ascending).
        uint32_t sub[CPT];
#pragma unroll
        for (int r = 0; r < CPT; ++r) {
            sub[r] = 0xffffffffu;
            if ((uint32_t)r * kFusedThreads + tid < listed) {
                sub[r] = linear_sub_bin(key_to_float(c[r].x), bin_scale, bstar);
                atomicAdd(&sub_hist[sub[r]], 1u);
            }
        }
        __syncthreads();
        if (tid < 64) {
            uint32_t s, r2;
            pick_bin<kSubBins>(sub_hist, rem, &s, &r2);
            if (lane == 0) { L.chosen[2] = s; L.chosen[3] = r2; }
        }
        __syncthreads();
        const uint32_t sstar = L.chosen[2], rem2 = L.chosen[3];
        uint32_t *list_key = L.sel.copies + kSubBins, *list_tile = L.equal_tile;
        uint32_t in_sub = 0;                     // bit r: my r-th candidate lies in the threshold's sub-bin
#pragma unroll
        for (int r = 0; r < CPT; ++r) {
            if (sub[r] != 0xffffffffu) {
                if (sub[r] > sstar) take_it(c[r].y);
                else if (sub[r] == sstar) {
                    in_sub |= 1u << r;
                    const uint32_t at = atomicAdd(&L.n_equal, 1u);
                    if (at < kFusedThreads) { list_key[at] = c[r].x; list_tile[at] = c[r].y; }
                }
            }
        }
        __syncthreads();
        const uint32_t nl = L.n_equal;
        if (nl <= kFusedThreads) {
            if ((uint32_t)tid < nl) {
                const uint32_t key = list_key[tid], tile = list_tile[tid];
                uint32_t ahead = 0;
                for (uint32_t i = 0; i < nl; ++i) {
                    const uint32_t ki = list_key[i];
                    ahead += (ki > key || (ki == key && list_tile[i] < tile)) ? 1u : 0u;
                }
                if (ahead < rem2) take_it(tile);
            }
        } else {
            __syncthreads();                     // the list is dropped: its memory serves the radix select
            rank_candidates(rem2, [&](auto f) {
#pragma unroll
                for (int r = 0; r < CPT; ++r)
                    if ((in_sub >> r) & 1u) f(c[r].x, c[r].y);
            }, take_it, L);
        }
    }
    above_before += before;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) above_before += (uint32_t)__shfl_xor((int)above_before, off, 64);
    if (lane == 0 && above_before != 0) atomicAdd(&L.n_before, above_before);
    __syncthreads();
    // the block's final words and rank-table entries: one group per thread of the first four wavefronts
    uint32_t lo = 0, hi = 0;
    if ((uint32_t)tid < GROUPS) { lo = L.words[2 * tid]; hi = L.words[2 * tid + 1]; }
    const uint32_t cnt = (uint32_t)__popc(lo) + (uint32_t)__popc(hi);
    const uint32_t incl = wave_incl_scan(cnt);
    if (lane == 63) L.wave_total[wave] = incl;
    __syncthreads();
    if ((uint32_t)tid < mygroups) {
        uint32_t rank = u * k + L.n_before + incl - cnt;     // every earlier unit holds exactly k wide tiles
        for (int w = 0; w < wave; ++w) rank += L.wave_total[w];
        ubitmap[group0 + tid] = ((uint64_t)hi << 32) | lo;
        uranks[group0 + tid] = rank;
    }
}

// A budget of exactly `lo` or `lo + 1` bits: every tile has the same width.  Bit map word and rank-table entry `w`.
__device__ __forceinline__ void constant_width_word(uint64_t w, uint32_t T, int all_wide, uint64_t *__restrict__ bitmap,
                                                    uint32_t *__restrict__ ranks)
{
    uint64_t bits = 0;
    if (all_wide) {
        const uint64_t left = (uint64_t)T - w * 64;
        bits = left >= 64 ? ~0ull : ((1ull << left) - 1ull);
    }
    bitmap[w] = bits;
    ranks[w] = all_wide ? (uint32_t)(w * 64) : 0u;
}

__global__ __launch_bounds__(256) void k_bitmap_const(uint32_t T, int all_wide, uint64_t *__restrict__ bitmap,
                                                      uint32_t *__restrict__ ranks)
{
    const uint64_t w = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (w < ((uint64_t)T + 63) / 64) constant_width_word(w, T, all_wide, bitmap, ranks);
}

// Header, zeroed section padding, zeroed histograms.
struct HeaderWords { uint32_t w[16]; };
struct PadList { uint64_t begin[5]; uint32_t len[5]; };

// With `const_words` != 0 it also writes the bit map and the rank table of a tensor whose tiles all have the same width
// (what k_bitmap_const does in a launch of its own).
__global__ __launch_bounds__(256) void k_prologue(uint8_t *__restrict__ packed, HeaderWords hdr, PadList pads,
                                                  uint32_t *__restrict__ zero_base, uint32_t zero_words,
                                                  uint32_t const_words, uint32_t T, int all_wide,
                                                  uint64_t *__restrict__ bitmap, uint32_t *__restrict__ ranks)
{
    const uint32_t gid = blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0) {
        if (threadIdx.x < 16) reinterpret_cast<uint32_t *>(packed)[threadIdx.x] = hdr.w[threadIdx.x];
        for (int s = 0; s < 5; ++s)
            if (threadIdx.x < pads.len[s]) packed[pads.begin[s] + threadIdx.x] = 0;
    }
    for (uint32_t i = gid; i < zero_words; i += gridDim.x * 256) zero_base[i] = 0u;
    for (uint32_t w = gid; w < const_words; w += gridDim.x * 256) constant_width_word(w, T, all_wide, bitmap, ranks);
}

}  // namespace tahq
