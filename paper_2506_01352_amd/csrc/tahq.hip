// TAH-Quant stage-boundary activation codec for gfx950: launch glue and C ABI.
//
// Paper sections implemented by the kernels this file launches: Sec. 3.1 (tiles of G contiguous
// channels), Sec. 3.2 Eq. 1-2 (entropy) and top-p% selection, Sec. 3.3 Eq. 3-4 (outlier test,
// pivot swap, Hadamard transform, asymmetric quantizer), Sec. 3.4 (byte stream), Alg. 1 step 5
// (dequantize); and, for the backward direction, Sec. 3.5 / Alg. 1 steps 6-7 with the appendix's gradient
// scaling (fixed-point compressor, tahq_naive_*).
//
// Numerics contract (identical results on any mapping of tiles to lanes):
//   * all arithmetic is IEEE binary32, no contraction (-ffp-contract=off); fused multiply-adds
//     only where written (__builtin_fmaf);
//   * sums over a tile use the adjacent-pair binary tree; an allocation tile of several quantization
//     tiles adds their sums from left to right;
//   * the Hadamard butterfly runs its stages h = 1, 2, ..., G/2 in that order;
//   * log(u) = e*ln2 + P(m) with (m, e) = frexp(u) and a fixed degree-5 polynomial;
//   * scale / zero-point are binary16, rounded outwards (up / down).
#include "tahq_common.hpp"
#include "tahq_select.hpp"
#include "tahq_stream_kernels.hpp"
#include "tahq_naive_kernels.hpp"
#include "tahq_naive.h"

#include <atomic>
#include <mutex>
#include <tuple>
#include <utility>

using namespace tahq;

// Built-in scratch of tahq_encode_noalloc: encoder workspace for callers that cannot provide one.  Every GPU
// the library runs on holds its own copy of this array, at its own address, until the process ends.
constexpr size_t kBuiltinScratchBytes = (size_t)TAHQ_NOALLOC_MAX_WORKSPACE;
static __device__ __align__(256) unsigned char scratch[kBuiltinScratchBytes];

namespace {

// Device address of `scratch` on every device that tahq_encode_noalloc has been called on.  In host code the
// array's name is only a handle for hipGetSymbolAddress: kernels are given the address kept here.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];


inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline uint32_t blocks_for(uint64_t threads) { return (uint32_t)((threads + 255) / 256); }

// Dispatch on the tile width G and on a dtype flag (bf16 or not) to a functor template.
template <template <int, bool> class F, typename... Args>
inline void dispatch(uint32_t G, bool bf16, Args... args)
{
    if (G == 8) { if (bf16) F<8, true>::run(args...); else F<8, false>::run(args...); }
    else if (G == 16) { if (bf16) F<16, true>::run(args...); else F<16, false>::run(args...); }
    else if (G == 32) { if (bf16) F<32, true>::run(args...); else F<32, false>::run(args...); }
    else if (G == 64) { if (bf16) F<64, true>::run(args...); else F<64, false>::run(args...); }
    else { if (bf16) F<128, true>::run(args...); else F<128, false>::run(args...); }
}

// Kernel launches of one call: each launch returns its own status (the thread's sticky "last error", which may
// belong to the caller's earlier work, is neither read nor cleared), and after a failure nothing more is enqueued.
struct Enqueue {
    hipStream_t stream;
    hipError_t status = hipSuccess;

    template <typename... P, typename... A>
    void operator()(void (*kernel)(P...), dim3 grid, dim3 block, A... args)
    {
        static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
        if (status != hipSuccess) return;
        std::tuple<P...> values(static_cast<P>(args)...);
        status = launch(kernel, grid, block, values, std::index_sequence_for<P...>{});
    }
    tahq_status result() const { return status == hipSuccess ? TAHQ_OK : TAHQ_ERR_HIP; }

private:
    template <typename... P, size_t... I>
    hipError_t launch(void (*kernel)(P...), dim3 grid, dim3 block, std::tuple<P...> &values, std::index_sequence<I...>)
    {
        void *ptrs[] = {static_cast<void *>(&std::get<I>(values))...};
        return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, 0, stream);
    }
};

// Grid of a persistent kernel: four times the workgroups that fit on the device at once (or fewer, if there
// are fewer batches).  Every workgroup still pipelines a few batches, and the hardware dispatcher evens
// out the load; a grid of exactly the resident count measured up to 30% slower.
// The resident count of a kernel is a property of the kernel and the device; it is looked up once per kernel and
// device (a query of the runtime, no stream operation: also legal while a stream is being captured) and kept
// in `cache`, one slot per device.
struct ResidentCache { std::atomic<uint32_t> per_device[kMaxDevices]; };

inline uint32_t resident_blocks(const void *kernel, int threads, ResidentCache &cache)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) dev = 0;
    const bool cached = dev < kMaxDevices;
    if (cached) {
        const uint32_t known = cache.per_device[dev].load(std::memory_order_relaxed);
        if (known) return known;
    }
    int cus = 256, per_cu = 1;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu <= 0) per_cu = 1;
    const uint32_t res = 4u * (uint32_t)cus * (uint32_t)per_cu;
    if (cached) cache.per_device[dev].store(res, std::memory_order_relaxed);
    return res;
}

template <int G, bool BF16>
struct LaunchEntropy {
    // hist != nullptr: also build the selection's first histogram, `bins` bins per ranking unit (units must be whole
    // batches): the keys' first radix digit if bin_scale == 0, the entropies' linear bins otherwise
    static void run(const void *d_in, float *d_H, uint32_t T, float eps_l1, float eps_log, uint32_t *hist,
                    uint32_t bins, float bin_scale, uint64_t n_per_unit, Enqueue *qp)
    {
        Enqueue &q = *qp;
        using B = Batch<G, BF16 ? 2 : 4>;
        const uint32_t nb = (T + B::TILES - 1) / B::TILES;
        static ResidentCache cache;
        const uint32_t res = resident_blocks(reinterpret_cast<const void *>(k_entropy<G, BF16>), B::TILES, cache);
        const uint32_t unit_batches = hist ? (uint32_t)(n_per_unit / B::TILES) : 1u;
        q(k_entropy<G, BF16>, dim3(nb < res ? nb : res), dim3(B::TILES), d_in, d_H, T,
                           eps_l1, eps_log, hist, unit_batches, bins, bin_scale);
    }
    static bool can_fuse_histogram(uint64_t n_per_unit) { return n_per_unit % Batch<G, BF16 ? 2 : 4>::TILES == 0; }
};

template <int G, bool BF16>
struct CanFuse {
    static void run(uint64_t n_per_unit, bool *out) { *out = LaunchEntropy<G, BF16>::can_fuse_histogram(n_per_unit); }
};

// `low`: the narrower of the two code widths, 1..7 (3: INT3/INT4).
template <int G, bool BF16>
struct LaunchQuantPack {
    template <int LOW>
    static void go(const void *d_in, uint8_t *packed, Layout lay, uint32_t T, float tau, float eps_ratio, Enqueue *qp)
    {
        Enqueue &q = *qp;
        using B = Batch<G, BF16 ? 2 : 4>;
        const uint32_t nb = (T + B::TILES - 1) / B::TILES;
        q(k_quant_pack<G, BF16, LOW>, dim3(nb), dim3(B::TILES), d_in, packed, lay, T, tau,
                           eps_ratio);
    }
    static void run(uint32_t low, const void *d_in, uint8_t *packed, Layout lay, uint32_t T, float tau, float eps_ratio,
                    Enqueue *qp)
    {
        switch (low) {
        case 1: go<1>(d_in, packed, lay, T, tau, eps_ratio, qp); break;
        case 2: go<2>(d_in, packed, lay, T, tau, eps_ratio, qp); break;
        case 3: go<3>(d_in, packed, lay, T, tau, eps_ratio, qp); break;
        case 4: go<4>(d_in, packed, lay, T, tau, eps_ratio, qp); break;
        case 5: go<5>(d_in, packed, lay, T, tau, eps_ratio, qp); break;
        case 6: go<6>(d_in, packed, lay, T, tau, eps_ratio, qp); break;
        default: go<7>(d_in, packed, lay, T, tau, eps_ratio, qp); break;
        }
    }
};

template <int G, bool BF16>
struct LaunchDecode {
    template <int LOW>
    static void go(const uint8_t *packed, void *d_out, Layout lay, uint32_t T, uint32_t total_wide, Enqueue *qp)
    {
        Enqueue &q = *qp;
        using B = Batch<G, BF16 ? 2 : 4>;
        const uint32_t nb = (T + B::TILES - 1) / B::TILES;
        static ResidentCache cache;
        const uint32_t res = resident_blocks(reinterpret_cast<const void *>(k_decode<G, BF16, LOW>), B::TILES, cache);
        q(k_decode<G, BF16, LOW>, dim3(nb < res ? nb : res), dim3(B::TILES), packed, d_out, lay,
                           T, total_wide);
    }
    static void run(uint32_t low, const uint8_t *packed, void *d_out, Layout lay, uint32_t T, uint32_t total_wide,
                    Enqueue *qp)
    {
        switch (low) {
        case 1: go<1>(packed, d_out, lay, T, total_wide, qp); break;
        case 2: go<2>(packed, d_out, lay, T, total_wide, qp); break;
        case 3: go<3>(packed, d_out, lay, T, total_wide, qp); break;
        case 4: go<4>(packed, d_out, lay, T, total_wide, qp); break;
        case 5: go<5>(packed, d_out, lay, T, total_wide, qp); break;
        case 6: go<6>(packed, d_out, lay, T, total_wide, qp); break;
        default: go<7>(packed, d_out, lay, T, total_wide, qp); break;
        }
    }
};

template <int G, bool BF16>
struct LaunchAllocEntropy {
    // Entropies of allocation tiles of m > 1 quantization tiles: one pass if a workgroup's batch holds whole
    // allocation tiles, otherwise two streaming passes over the tensor.
    static void run(const void *d_in, float *d_H, float *part, float *inv_norm, uint32_t T, uint32_t m, float eps_l1,
                    float eps_log, Enqueue *qp)
    {
        Enqueue &q = *qp;
        using B = Batch<G, BF16 ? 2 : 4>;
        const uint32_t nb = (T + B::TILES - 1) / B::TILES;
        const uint32_t n_alloc = T / m;
        if (B::TILES % m == 0) {
            q(k_alloc_entropy<G, BF16>, dim3(nb), dim3(B::TILES), d_in, d_H, T, m, eps_l1,
                               eps_log);
            return;
        }
        q(k_tile_partial<G, BF16, false>, dim3(nb), dim3(B::TILES), d_in,
                           (const float *)nullptr, part, T, m, eps_log);
        q(k_alloc_reduce<false>, dim3(blocks_for(n_alloc)), dim3(256), (const float *)part, (const float *)nullptr,
                           inv_norm, n_alloc, m, eps_l1);
        q(k_tile_partial<G, BF16, true>, dim3(nb), dim3(B::TILES), d_in,
                           (const float *)inv_norm, part, T, m, eps_log);
        q(k_alloc_reduce<true>, dim3(blocks_for(n_alloc)), dim3(256), (const float *)part, (const float *)inv_norm,
                           d_H, n_alloc, m, eps_l1);
    }
};

// Entropy of every quantization tile; with `hist`, also the selection's first histogram (the caller has checked
// that the ranking units are whole batches).
void launch_entropy(const Shape &s, const tahq_config *cfg, const void *d_in, float *d_H, uint32_t *hist, uint32_t bins,
                    float bin_scale, Enqueue *qp)
{
    dispatch<LaunchEntropy>(s.G, s.dtype == TAHQ_BF16, d_in, d_H, (uint32_t)s.T, cfg->eps_l1, cfg->eps_log, hist, bins,
                            bin_scale, s.n, qp);
}

// ---- backward-pass fixed-point compressor

struct NaiveShape {
    uint64_t N;          // elements
    uint32_t nchunks;    // chunks of 32 elements
    uint32_t bits, dtype;
    uint64_t total;      // stream bytes
};

tahq_status make_naive_shape(const tahq_naive_config *c, NaiveShape *s)
{
    if (!c) return TAHQ_ERR_NULL;
    if (c->struct_size != sizeof(tahq_naive_config)) return TAHQ_ERR_INVALID_ARG;
    if (c->batch == 0 || c->seq == 0 || c->hidden == 0 || c->hidden % kNaiveChunk != 0) return TAHQ_ERR_INVALID_ARG;
    if (c->dtype > TAHQ_BF16 || c->bits < 2 || c->bits > 16) return TAHQ_ERR_INVALID_ARG;
    if (!(c->scale > 0.0f) || c->scale > 3.4028234663852886e38f) return TAHQ_ERR_INVALID_ARG;
    const uint64_t N = (uint64_t)c->batch * c->seq * c->hidden;
    if (N > (1ull << 36)) return TAHQ_ERR_INVALID_ARG;
    s->N = N;
    s->nchunks = (uint32_t)(N / kNaiveChunk);
    s->bits = c->bits;
    s->dtype = c->dtype;
    s->total = 64 + N * c->bits / 8;
    return TAHQ_OK;
}

template <int BITS>
void launch_naive_encode(bool bf16, const void *d_in, uint8_t *packed, const NaiveHeader &hdr, uint32_t nchunks,
                         float scale, Enqueue *qp)
{
    Enqueue &q = *qp;
    const dim3 grid((nchunks + kNaiveChunks - 1) / kNaiveChunks), block(kNaiveChunks);
    if (bf16) q(k_naive_encode<BITS, true>, grid, block, d_in, packed, hdr, nchunks, scale);
    else q(k_naive_encode<BITS, false>, grid, block, d_in, packed, hdr, nchunks, scale);
}

template <int BITS>
void launch_naive_decode(bool out_bf16, const uint8_t *packed, void *d_out, uint32_t nchunks, float inv_scale,
                         Enqueue *qp)
{
    Enqueue &q = *qp;
    const dim3 grid((nchunks + kNaiveChunks - 1) / kNaiveChunks), block(kNaiveChunks);
    if (out_bf16) q(k_naive_decode<BITS, true>, grid, block, packed, d_out, nchunks, inv_scale);
    else q(k_naive_decode<BITS, false>, grid, block, packed, d_out, nchunks, inv_scale);
}

// Every supported code width, for the switch over the run-time width.
#define TAHQ_NAIVE_WIDTHS(X) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16)

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
    return s.kA;
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
    Enqueue q{(hipStream_t)stream};
    launch_entropy(s, cfg, d_in, d_entropy, nullptr, 0u, 0.0f, &q);
    return q.result();
}

tahq_status tahq_alloc_tile_entropy(const tahq_config *cfg, const void *d_in, float *d_entropy, void *d_workspace,
                                    size_t workspace_capacity, tahq_stream stream)
{
    Shape s;
    tahq_status rc = make_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    if (!d_in || !d_entropy) return TAHQ_ERR_NULL;
    if (misaligned(d_in) || misaligned(d_entropy)) return TAHQ_ERR_MISALIGNED;
    Enqueue q{(hipStream_t)stream};
    if (s.m == 1) {
        launch_entropy(s, cfg, d_in, d_entropy, nullptr, 0u, 0.0f, &q);
    } else {
        if (!d_workspace) return TAHQ_ERR_NULL;
        Workspace ws;
        make_workspace(s, &ws);
        if (workspace_capacity < ws.total) return TAHQ_ERR_WORKSPACE_TOO_SMALL;
        if (misaligned(d_workspace)) return TAHQ_ERR_MISALIGNED;
        uint8_t *wsb = static_cast<uint8_t *>(d_workspace);
        dispatch<LaunchAllocEntropy>(s.G, s.dtype == TAHQ_BF16, d_in, d_entropy,
                                     reinterpret_cast<float *>(wsb + ws.part),
                                     reinterpret_cast<float *>(wsb + ws.inv_norm), (uint32_t)s.T, s.m, cfg->eps_l1,
                                     cfg->eps_log, &q);
    }
    return q.result();
}

tahq_status tahq_encode_phases(const tahq_config *cfg, const void *d_in, void *d_packed, size_t packed_capacity,
                               void *d_workspace, size_t workspace_capacity, uint32_t phases, tahq_stream stream)
{
    const bool multi_launch = (phases & TAHQ_SELECT_MULTI_LAUNCH) != 0;
    phases &= ~(uint32_t)TAHQ_SELECT_MULTI_LAUNCH;
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
    // the selection kernels of large ranking units put the unit into the grid's second dimension
    if (s.kA != 0 && s.kA != s.nA && s.U > 65535u && (s.nA > kSmallUnitMaxKeys || multi_launch))
        return TAHQ_ERR_UNSUPPORTED;

    Enqueue q{(hipStream_t)stream};
    uint8_t *packed = static_cast<uint8_t *>(d_packed);
    uint8_t *wsb = static_cast<uint8_t *>(d_workspace);
    uint64_t *bitmap = reinterpret_cast<uint64_t *>(packed + lay.bitmap);
    uint32_t *ranks = reinterpret_cast<uint32_t *>(packed + lay.ranks);
    const bool select = s.kA != 0 && s.kA != s.nA;
    const bool wide = s.m > 1;     // allocation tiles of several quantization tiles
    // ranking units that one workgroup can hold are ranked in a single launch
    const bool small_units = select && s.nA <= kSmallUnitMaxKeys && !multi_launch;

    // header, section padding, selection scratch
    HeaderWords hdr;
    memset(&hdr, 0, sizeof hdr);
    hdr.w[0] = 0x51484154u;   // "TAHQ"
    hdr.w[1] = 1;
    hdr.w[2] = s.dtype; hdr.w[3] = s.B; hdr.w[4] = s.S; hdr.w[5] = s.C; hdr.w[6] = s.G; hdr.w[7] = s.scope;
    hdr.w[8] = (uint32_t)s.kA;
    hdr.w[14] = s.A;
    hdr.w[15] = s.low;
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
    const bool histograms = select && !small_units;
    const uint32_t zero_words = histograms ? (uint32_t)(ws.zero_bytes / 4) : 0u;
    // a tensor whose tiles all have the same width needs no selection: its bit map and rank table are constants, which
    // the prologue writes as well when the caller asks for both phases at once
    const bool const_in_prologue = !select && (phases & TAHQ_PHASE_PROLOGUE) && (phases & TAHQ_PHASE_SELECT);
    if (phases & TAHQ_PHASE_PROLOGUE) {
        const uint32_t const_words = const_in_prologue ? (uint32_t)words64 : 0u;
        const uint32_t blocks = histograms ? 32u : (const_words ? (blocks_for(words64) < 256u ? blocks_for(words64) : 256u) : 1u);
        q(k_prologue, dim3(blocks), dim3(256), packed, hdr, pads, reinterpret_cast<uint32_t *>(wsb + ws.hist0), zero_words,
          const_words, (uint32_t)s.T, s.kA == s.nA ? 1 : 0, bitmap, ranks);
    }

    if (select) {
        float *H = reinterpret_cast<float *>(wsb + ws.keys);
        uint32_t *hist0 = reinterpret_cast<uint32_t *>(wsb + ws.hist0);
        uint32_t *coarse = reinterpret_cast<uint32_t *>(wsb + ws.coarse);
        uint32_t *partial = reinterpret_cast<uint32_t *>(wsb + ws.partial);
        uint32_t *state = reinterpret_cast<uint32_t *>(wsb + ws.state);
        uint32_t *seg = reinterpret_cast<uint32_t *>(wsb + ws.seg);
        uint8_t *sel = wsb + ws.sel;
        // the entropy kernel builds the selection's first histogram itself when units are whole batches
        bool whole_batches = false;
        if (!wide && !small_units) dispatch<CanFuse>(s.G, s.dtype == TAHQ_BF16, s.n, &whole_batches);
        // Large units that start on 64-tile boundaries are ranked in one launch from a histogram of linear bins;
        // everything else (and every unit when the caller forces it) by the multi-launch radix select.
        const bool fused_select = whole_batches && !multi_launch && s.n % 64 == 0;
        const bool fused = whole_batches && !fused_select;       // first radix digit folded into the entropy kernel
        uint32_t *lin_hist = reinterpret_cast<uint32_t *>(wsb + ws.lin_hist);
        // bins of width ln(A) / kLinBins: the entropy of A channels lies in [0, ln A]
        const float bin_scale = (float)((double)kLinBins / __builtin_log((double)s.A));
        if (phases & TAHQ_PHASE_ENTROPY) {
            if (wide)
                dispatch<LaunchAllocEntropy>(s.G, s.dtype == TAHQ_BF16, d_in, H, reinterpret_cast<float *>(wsb + ws.part),
                                             reinterpret_cast<float *>(wsb + ws.inv_norm), (uint32_t)s.T, s.m,
                                             cfg->eps_l1, cfg->eps_log, &q);
            else if (fused_select)
                launch_entropy(s, cfg, d_in, H, lin_hist, kLinBins, bin_scale, &q);
            else
                launch_entropy(s, cfg, d_in, H, fused ? hist0 : (uint32_t *)nullptr, kDigit0Bins, 0.0f, &q);
        }
        if ((phases & TAHQ_PHASE_SELECT) && fused_select) {
            const dim3 grid((uint32_t)((s.n + kFusedKeysPerBlock - 1) / kFusedKeysPerBlock), s.U);
            uint32_t *fused_state = reinterpret_cast<uint32_t *>(wsb + ws.fused);
            uint2 *cand = reinterpret_cast<uint2 *>(wsb + ws.cand);
            uint32_t *block_above = reinterpret_cast<uint32_t *>(wsb + ws.block_above);
            q(k_select_classify, grid, dim3(kFusedThreads), (const float *)H, (uint32_t)s.n,
                               (uint32_t)s.k, bin_scale, (const uint32_t *)lin_hist, fused_state, cand, block_above,
                               bitmap);
            q(k_select_resolve, grid, dim3(kFusedThreads), (const float *)H, (uint32_t)s.n,
                               (uint32_t)s.k, bin_scale, (const uint32_t *)lin_hist, (const uint32_t *)fused_state,
                               (const uint2 *)cand, (const uint32_t *)block_above, bitmap, ranks);
        } else
        if ((phases & TAHQ_PHASE_SELECT) && small_units) {
            const uint32_t n32 = (uint32_t)s.nA, k32 = (uint32_t)s.kA;
            const int aligned = (!wide && s.n % 64 == 0) ? 1 : 0;
            uint32_t *ranks_a = reinterpret_cast<uint32_t *>(wsb + ws.ranks_a);
            uint32_t *rank_out = wide ? ranks_a : ranks;
            const dim3 grid(s.U), block(kSmallUnitThreads);
            if (n32 <= 16 * kSmallUnitThreads)
                q(k_select_small<16>, grid, block, (const float *)H, n32, k32, bitmap, rank_out, sel, aligned);
            else
                q(k_select_small<32>, grid, block, (const float *)H, n32, k32, bitmap, rank_out, sel, aligned);
            if (wide)
                q(k_expand_alloc, dim3(blocks_for(words64 * 64)), dim3(256),
                                   (const uint8_t *)sel, (const uint32_t *)ranks_a, (uint32_t)s.T, s.m, bitmap, ranks);
            else if (!aligned)
                q(k_bitmap_pack, dim3(blocks_for(words64 * 64)), dim3(256),
                                   (const uint8_t *)sel, (uint32_t)s.T, bitmap);
        } else if (phases & TAHQ_PHASE_SELECT) {
            // the selection ranks allocation tiles; with A = G they are the stream's tiles
            const uint32_t n32 = (uint32_t)s.nA, k32 = (uint32_t)s.kA;
            const dim3 rgrid(ws.hb, s.U);
            if (!fused)
                q(k_radix_pass<0, 8>, rgrid, dim3(256), (const float *)H, n32, k32, hist0, coarse, partial, state);
            q(k_radix_pass<1, 0>, rgrid, dim3(256), (const float *)H, n32, k32, hist0, coarse, partial, state);
            q(k_radix_pass<2, 0>, rgrid, dim3(256), (const float *)H, n32, k32, hist0, coarse, partial, state);
            const uint32_t sb = (ws.nseg + 3) / 4;
            q(k_seg_count, dim3(sb, s.U), dim3(256), (const float *)H, n32, ws.nseg,
                               (const uint32_t *)coarse, (const uint32_t *)partial, ws.hb, state, seg);
            const int aligned = (!wide && s.n % 64 == 0) ? 1 : 0;
            uint32_t *ranks_a = reinterpret_cast<uint32_t *>(wsb + ws.ranks_a);
            q(k_assign, dim3(sb, s.U), dim3(256), (const float *)H, n32, k32, ws.nseg,
                               (const uint32_t *)state, (const uint32_t *)seg, bitmap, wide ? ranks_a : ranks, sel,
                               aligned);
            if (wide)
                q(k_expand_alloc, dim3(blocks_for(words64 * 64)), dim3(256),
                                   (const uint8_t *)sel, (const uint32_t *)ranks_a, (uint32_t)s.T, s.m, bitmap, ranks);
            else if (!aligned)
                q(k_bitmap_pack, dim3(blocks_for(words64 * 64)), dim3(256),
                                   (const uint8_t *)sel, (uint32_t)s.T, bitmap);
        }
    } else if ((phases & TAHQ_PHASE_SELECT) && !const_in_prologue) {
        q(k_bitmap_const, dim3(blocks_for(words64)), dim3(256), (uint32_t)s.T,
                           s.kA == s.nA ? 1 : 0, bitmap, ranks);
    }

    if (phases & TAHQ_PHASE_QUANT) {
        dispatch<LaunchQuantPack>(s.G, s.dtype == TAHQ_BF16, s.low, d_in, packed, lay, (uint32_t)s.T, cfg->tau,
                                  cfg->eps_ratio, &q);
    }
    return q.result();
}

tahq_status tahq_encode(const tahq_config *cfg, const void *d_in, void *d_packed, size_t packed_capacity,
                        void *d_workspace, size_t workspace_capacity, tahq_stream stream)
{
    return tahq_encode_phases(cfg, d_in, d_packed, packed_capacity, d_workspace, workspace_capacity,
                              TAHQ_PHASE_ALL, stream);
}

tahq_status tahq_encode_noalloc(const tahq_config *cfg, const void *d_in, void *d_packed, size_t packed_capacity,
                                tahq_stream stream)
{
    Shape s;
    tahq_status rc = make_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    Workspace ws;
    make_workspace(s, &ws);
    if (ws.total > kBuiltinScratchBytes) return TAHQ_ERR_TOO_LARGE;
    if (!d_in || !d_packed) return TAHQ_ERR_NULL;
    Layout lay;
    make_layout(s, &lay);
    if (packed_capacity < lay.total) return TAHQ_ERR_BUFFER_TOO_SMALL;
    if (misaligned(d_in) || misaligned(d_packed)) return TAHQ_ERR_MISALIGNED;
    // the current device's copy of the built-in scratch: looked up once per device, with that device current
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TAHQ_ERR_HIP;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        ptr = g_scratch_ptr[dev];
        if (!ptr) {
            if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TAHQ_ERR_HIP;
            g_scratch_ptr[dev] = ptr;
        }
    }
    // what must start at zero in there (the selection's histograms and state) is cleared by the encoder's
    // first kernel, as it is in a caller's workspace
    return tahq_encode_phases(cfg, d_in, d_packed, packed_capacity, ptr, kBuiltinScratchBytes, TAHQ_PHASE_ALL, stream);
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
    Enqueue q{(hipStream_t)stream};
    dispatch<LaunchDecode>(s.G, out_dtype == TAHQ_BF16, s.low, static_cast<const uint8_t *>(d_packed), d_out, lay,
                           (uint32_t)s.T, (uint32_t)(s.U * s.k), &q);
    return q.result();
}

// ---- sample-wise use: a run of samples as a tensor of its own

namespace {
// The configuration of samples [first, first + count) taken as a tensor [count, seq, hidden], and the byte offset
// of the first of them in the whole tensor (element size `esize`).
tahq_status samples_config(const tahq_config *cfg, uint32_t first, uint32_t count, uint32_t esize, tahq_config *sub,
                           uint64_t *offset)
{
    Shape s;
    tahq_status rc = make_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    if (s.scope != 0 || count == 0 || first >= s.B || count > s.B - first) return TAHQ_ERR_INVALID_ARG;
    memset(sub, 0, sizeof *sub);
    memcpy(sub, cfg, cfg->struct_size);          // older, shorter layouts: the missing fields stay 0
    sub->batch = count;
    *offset = (uint64_t)first * s.S * s.C * esize;
    return TAHQ_OK;
}
}  // namespace

size_t tahq_samples_packed_size(const tahq_config *cfg, uint32_t count)
{
    tahq_config sub;
    uint64_t off;
    if (samples_config(cfg, 0, count, 1, &sub, &off) != TAHQ_OK) return 0;
    return tahq_packed_size(&sub);
}

size_t tahq_samples_workspace_size(const tahq_config *cfg, uint32_t count)
{
    tahq_config sub;
    uint64_t off;
    if (samples_config(cfg, 0, count, 1, &sub, &off) != TAHQ_OK) return 0;
    return tahq_workspace_size(&sub);
}

tahq_status tahq_encode_samples(const tahq_config *cfg, uint32_t first, uint32_t count, const void *d_in, void *d_packed,
                                size_t packed_capacity, void *d_workspace, size_t workspace_capacity, tahq_stream stream)
{
    if (!cfg) return TAHQ_ERR_NULL;
    tahq_config sub;
    uint64_t off;
    tahq_status rc = samples_config(cfg, first, count, cfg->dtype == TAHQ_BF16 ? 2u : 4u, &sub, &off);
    if (rc != TAHQ_OK) return rc;
    if (!d_in) return TAHQ_ERR_NULL;
    return tahq_encode(&sub, static_cast<const uint8_t *>(d_in) + off, d_packed, packed_capacity, d_workspace,
                       workspace_capacity, stream);
}

tahq_status tahq_decode_samples(const tahq_config *cfg, uint32_t first, uint32_t count, const void *d_packed,
                                size_t packed_bytes, void *d_out, uint32_t out_dtype, tahq_stream stream)
{
    if (!cfg) return TAHQ_ERR_NULL;
    if (out_dtype > TAHQ_BF16) return TAHQ_ERR_INVALID_ARG;
    tahq_config sub;
    uint64_t off;
    tahq_status rc = samples_config(cfg, first, count, out_dtype == TAHQ_BF16 ? 2u : 4u, &sub, &off);
    if (rc != TAHQ_OK) return rc;
    if (!d_out) return TAHQ_ERR_NULL;
    return tahq_decode(&sub, d_packed, packed_bytes, static_cast<uint8_t *>(d_out) + off, out_dtype, nullptr, 0, stream);
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
    cfg->alloc_tile = w[14];
    cfg->low_bits = w[15];
    Shape s;
    tahq_status rc = make_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    return s.kA == w[8] ? TAHQ_OK : TAHQ_ERR_INVALID_ARG;
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
    case TAHQ_ERR_TOO_LARGE: return "configuration needs more scratch than the built-in buffer of tahq_encode_noalloc holds";
    }
    return "unknown status";
}

uint32_t tahq_version(void) { return (1u << 16) | 1u; }

void tahq_naive_config_default(tahq_naive_config *cfg)
{
    if (!cfg) return;
    memset(cfg, 0, sizeof *cfg);
    cfg->struct_size = (uint32_t)sizeof *cfg;
    cfg->dtype = TAHQ_BF16;
    cfg->bits = 8;
    cfg->scale = 1.0f;
}

size_t tahq_naive_packed_size(const tahq_naive_config *cfg)
{
    NaiveShape s;
    if (make_naive_shape(cfg, &s) != TAHQ_OK) return 0;
    return (size_t)s.total;
}

tahq_status tahq_naive_encode(const tahq_naive_config *cfg, const void *d_in, void *d_packed, size_t packed_capacity,
                              tahq_stream stream)
{
    NaiveShape s;
    tahq_status rc = make_naive_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    if (!d_in || !d_packed) return TAHQ_ERR_NULL;
    if (packed_capacity < s.total) return TAHQ_ERR_BUFFER_TOO_SMALL;
    if (misaligned(d_in) || misaligned(d_packed)) return TAHQ_ERR_MISALIGNED;
    NaiveHeader hdr;
    memset(&hdr, 0, sizeof hdr);
    hdr.w[0] = 0x4e484154u;   // "TAHN"
    hdr.w[1] = 1;
    hdr.w[2] = cfg->dtype; hdr.w[3] = cfg->batch; hdr.w[4] = cfg->seq; hdr.w[5] = cfg->hidden; hdr.w[6] = cfg->bits;
    memcpy(&hdr.w[7], &cfg->scale, 4);
    uint8_t *packed = static_cast<uint8_t *>(d_packed);
    const bool bf16 = cfg->dtype == TAHQ_BF16;
    Enqueue q{(hipStream_t)stream};
    switch (cfg->bits) {
#define X(B) case B: launch_naive_encode<B>(bf16, d_in, packed, hdr, s.nchunks, cfg->scale, &q); break;
        TAHQ_NAIVE_WIDTHS(X)
#undef X
    default: return TAHQ_ERR_INVALID_ARG;
    }
    return q.result();
}

tahq_status tahq_naive_decode(const tahq_naive_config *cfg, const void *d_packed, size_t packed_bytes, void *d_out,
                              uint32_t out_dtype, tahq_stream stream)
{
    NaiveShape s;
    tahq_status rc = make_naive_shape(cfg, &s);
    if (rc != TAHQ_OK) return rc;
    if (out_dtype > TAHQ_BF16) return TAHQ_ERR_INVALID_ARG;
    if (!d_packed || !d_out) return TAHQ_ERR_NULL;
    if (packed_bytes < s.total) return TAHQ_ERR_BUFFER_TOO_SMALL;
    if (misaligned(d_packed) || misaligned(d_out)) return TAHQ_ERR_MISALIGNED;
    const float inv_scale = 1.0f / cfg->scale;      // rounded once, on the host
    const uint8_t *packed = static_cast<const uint8_t *>(d_packed);
    Enqueue q{(hipStream_t)stream};
    switch (cfg->bits) {
#define X(B) case B: launch_naive_decode<B>(out_dtype == TAHQ_BF16, packed, d_out, s.nchunks, inv_scale, &q); break;
        TAHQ_NAIVE_WIDTHS(X)
#undef X
    default: return TAHQ_ERR_INVALID_ARG;
    }
    return q.result();
}

}  // extern "C"

