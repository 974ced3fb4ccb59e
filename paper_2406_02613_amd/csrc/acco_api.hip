// Host side of the C ABI declared in include/acco.h: argument validation, host
// counter bookkeeping, folding of the AdamW scalars, launch geometry.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <type_traits>

#include "../../include/acco.h"
#include "kernels.hpp"

#define ACCO_API extern "C" __attribute__((visibility("default")))

namespace {

using namespace acco;

// ------------------------------------------------------------------ launch shapes

// threads, vectors in flight, workgroups per CU and the resident-wavefront bound of one entry
// point, packed into one word so that a launch always sees a consistent set
struct LaunchShape {
    int threads;
    int vectors;    // U: 16-byte vectors per thread per array in flight
    int wg_per_cu;
    int resident;   // wavefronts resident per CU at most (0 = hardware limit)
};

inline uint64_t pack_shape(const LaunchShape& s)
{
    return (uint64_t)(uint16_t)s.threads | ((uint64_t)(uint8_t)s.vectors << 16) |
           ((uint64_t)(uint8_t)s.wg_per_cu << 24) | ((uint64_t)(uint8_t)s.resident << 32);
}

inline LaunchShape unpack_shape(uint64_t w)
{
    return LaunchShape{(int)(w & 0xFFFF), (int)((w >> 16) & 0xFF), (int)((w >> 24) & 0xFF),
                       (int)((w >> 32) & 0xFF)};
}

enum Entry {
    kAccumulate = 0,
    kCast,
    kReduce,
    kEstimate,
    kCommit,
    kAccumulatePublish,
    kReduceEstimate,
    kReduceCommit,
    kSgd,
    kStash,
    kSecond,
    kProbe,
    kEntries
};

// One wavefront per workgroup, one vector per thread: the fastest shape measured for every
// entry point at 875M elements (64 > 256 > 512 > 128 threads; looping variants slower still).
// Last column: wavefronts resident per CU at most.  The kernels that stream many arrays run
// faster with fewer wavefronts in flight than the hardware would admit (32): enough bytes are
// outstanding to cover the memory latency with 8-12 of them, and fewer concurrent wavefronts
// keep fewer DRAM pages open at a time.  Values from sweeps at 31M, 125M and 875M elements
// (same optimum at all three; no effect on cache-resident sizes).
constexpr LaunchShape kDefaults[kEntries] = {
    {64, 1, 0, 24},  // accumulate          (+1-2 %)
    {64, 1, 0, 0},   // cast                (any bound is slower)
    {64, 1, 0, 16},  // reduce              (+3 %)
    {64, 1, 0, 12},  // estimate            (+8 %)
    {64, 1, 0, 8},   // commit              (+5 %; 7 is over the edge: -5 %)
    {64, 1, 0, 24},  // accumulate_publish  (+1 %)
    {64, 1, 0, 10},  // reduce_estimate     (+6 %)
    {64, 1, 0, 9},   // reduce_commit       (+3 %)
    {64, 1, 0, 16},  // sgd                 (+2-3 %)
    {64, 1, 0, 0},   // stash               (no gain inside a round)
    {64, 1, 0, 18},  // second              (+4 % with bf16 output; fp32 output: unbounded)
    {64, 1, 0, 0},   // probe
};

std::atomic<uint64_t> g_shape[kEntries];

void reset_shapes()
{
    for (int e = 0; e < kEntries; ++e)
        g_shape[e].store(pack_shape(kDefaults[e]), std::memory_order_relaxed);
}

// the settings hold their defaults before any entry point can run
[[maybe_unused]] const bool g_shapes_ready = (reset_shapes(), true);

const char* const kEntryNames[kEntries] = {"accumulate",         "cast",            "reduce",
                                           "estimate",           "commit",          "accumulate_publish",
                                           "reduce_estimate",    "reduce_commit",   "sgd",
                                           "stash",              "second",          "probe"};

int cu_count()
{
    static std::atomic<int> cached[64];
    int                     dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int c = cached[dev].load(std::memory_order_relaxed);
    if (c == 0) {
        if (hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            c <= 0)
            c = 256;
        cached[dev].store(c, std::memory_order_relaxed);
    }
    return c;
}

struct Geometry {
    int      threads;
    int      vectors;
    int64_t  tiles;
    dim3     grid;
    unsigned lds_bytes;  // reserved (unused) LDS per workgroup: bounds the resident workgroups
};

constexpr int kLdsPerCu   = 160 * 1024;  // gfx950
constexpr int kLdsGranule = 1280;

// LDS reservation that lets exactly `groups` workgroups share a compute unit.
unsigned lds_for_groups(int groups)
{
    return (unsigned)(kLdsPerCu / groups / kLdsGranule * kLdsGranule);
}

Geometry geometry(Entry e, int64_t nvec, bool bounded, int rows = 1, int max_vectors = 4)
{
    const LaunchShape shape = unpack_shape(g_shape[e].load(std::memory_order_relaxed));
    Geometry          g;
    g.threads = shape.threads;
    // max_vectors == 0: an Op that only exists as the flat kernel - one vector per thread and no
    // cap on the workgroups, whatever the entry's shape says
    g.vectors = max_vectors == 0 ? 1 : shape.vectors > max_vectors ? max_vectors : shape.vectors;
    const int     per_cu = max_vectors == 0 ? 0 : shape.wg_per_cu;
    const int64_t tile   = (int64_t)g.threads * g.vectors;
    g.tiles              = (nvec + tile - 1) / tile;
    const int64_t want   = g.tiles < 1 ? 1 : g.tiles;  // the scalar tail still needs workgroup 0
    // a dispatch holds fewer than 2^32 work-items per dimension; shards too long for one
    // workgroup per tile fall back to the looping kernel
    const int64_t most   = (((int64_t)1 << 32) - 1) / g.threads;
    const int64_t asked  = per_cu > 0 ? (int64_t)per_cu * cu_count() : most;
    const int64_t cap    = asked < most ? asked : most;
    g.grid               = dim3((unsigned)(want < cap ? want : cap), (unsigned)rows);
    const int resident   = shape.resident;
    const int groups     = resident / (g.threads / 64);       // workgroups per CU
    g.lds_bytes = (bounded && resident > 0) ? lds_for_groups(groups < 3 ? 3 : groups) : 0u;
    return g;
}

// Launch of an Op source (Single<Op>: one Op; Batch<Op>: `rows` workers, one Op each, built on
// the device from a pointer table) over n elements per row.
// bounded = false: ignore the entry's bound on resident wavefronts (kernels that write more
// than they read want the full occupancy)
template <class Op, class = void>
struct MaxVectors {
    static constexpr int value = 4;
};
template <class Op>
struct MaxVectors<Op, std::void_t<decltype(Op::kMaxVectors)>> {
    static constexpr int value = Op::kMaxVectors;
};

template <class Src>
int launch_source(Entry e, const Src& src, int rows, int64_t n, hipStream_t stream, bool bounded)
{
    typedef typename Src::Op Op;
    constexpr int  kMaxV = MaxVectors<Op>::value;
    const int64_t  nvec  = n / Op::kElems;
    const Geometry g     = geometry(e, nvec, bounded, rows, kMaxV);
    if (g.vectors == 1 && (int64_t)g.grid.x >= g.tiles) {
        hipLaunchKernelGGL((flat_kernel<Src>), g.grid, dim3(g.threads), g.lds_bytes, stream, src, nvec,
                           n);
        return hipGetLastError() == hipSuccess ? ACCO_OK : ACCO_ERR_DEVICE;
    }
    if constexpr (kMaxV == 0) return ACCO_ERR_DEVICE;  // flat only, and too long for one dispatch
    if (g.vectors == 1) {
        if constexpr (kMaxV >= 1)
            hipLaunchKernelGGL((stream_kernel<1, Src>), g.grid, dim3(g.threads), g.lds_bytes, stream, src,
                               nvec, g.tiles, n);
    } else if (g.vectors == 2) {
        if constexpr (kMaxV >= 2)
            hipLaunchKernelGGL((stream_kernel<2, Src>), g.grid, dim3(g.threads), g.lds_bytes, stream, src,
                               nvec, g.tiles, n);
    } else {
        if constexpr (kMaxV >= 4)
            hipLaunchKernelGGL((stream_kernel<4, Src>), g.grid, dim3(g.threads), g.lds_bytes, stream, src,
                               nvec, g.tiles, n);
    }
    return hipGetLastError() == hipSuccess ? ACCO_OK : ACCO_ERR_DEVICE;
}

// Would a launch of entry e over n elements (4 per vector) run as flat_kernel?  With the
// entry's default shape it does, for any n the library accepts per dispatch.
bool flat_applies(Entry e, int64_t n)
{
    const Geometry g = geometry(e, n / 4, true);
    return g.vectors == 1 && (int64_t)g.grid.x >= g.tiles;
}

template <class Op>
int launch(Entry e, const Op& op, int64_t n, hipStream_t stream, bool bounded = true)
{
    return launch_source(e, Single<Op>{op}, 1, n, stream, bounded);
}

// workers [0, count) of the three pointer columns, kBatchMax per launch
template <class Op>
int launch_batch(Entry e, void* const* a, const void* const* b, const void* const* c, int count,
                 int64_t n, hipStream_t stream, const typename Op::Shared& shared = {},
                 bool bounded = true)
{
    for (int w0 = 0; w0 < count; w0 += kBatchMax) {
        const int rows = count - w0 < kBatchMax ? count - w0 : kBatchMax;
        Batch<Op> src;
        std::memset(&src.tab, 0, sizeof src.tab);
        src.shared = shared;
        for (int r = 0; r < rows; ++r) {
            src.tab.a[r] = a[w0 + r];
            src.tab.b[r] = b != nullptr ? b[w0 + r] : nullptr;
            src.tab.c[r] = c != nullptr ? c[w0 + r] : nullptr;
        }
        if (int rc = launch_source(e, src, rows, n, stream, bounded)) return rc;
    }
    return ACCO_OK;
}

// ------------------------------------------------------------------ validation helpers

inline bool aligned16(const void* p)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

inline bool overlap(const void* a, int64_t a_bytes, const void* b, int64_t b_bytes)
{
    if (a == nullptr || b == nullptr || a_bytes <= 0 || b_bytes <= 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + (uintptr_t)b_bytes && b0 < a0 + (uintptr_t)a_bytes;
}

inline int check_n(int64_t n)
{
    return (n < 0 || n > ACCO_MAX_ELEMS) ? ACCO_ERR_SIZE : ACCO_OK;
}

inline bool finite_nonneg(double x)
{
    return std::isfinite(x) && x >= 0.0;
}

int check_hyper(const acco_adamw_t* hp, int64_t step, int64_t total_count)
{
    if (hp == nullptr) return ACCO_ERR_NULL;
    if (!finite_nonneg(hp->lr) || !finite_nonneg(hp->eps) || !finite_nonneg(hp->weight_decay))
        return ACCO_ERR_ARG;
    if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0) || !(hp->beta2 >= 0.0 && hp->beta2 < 1.0))
        return ACCO_ERR_ARG;
    if (step < 0 || step == std::numeric_limits<int64_t>::max() || total_count < 1)
        return ACCO_ERR_ARG;
    return ACCO_OK;
}

// base + sum(counts) with overflow and sign checks
int sum_counts(const int64_t* counts, int workers, int64_t base, int64_t* out)
{
    if (base < 0) return ACCO_ERR_ARG;
    int64_t t = base;
    for (int w = 0; w < workers; ++w) {
        if (counts[w] < 0) return ACCO_ERR_ARG;
        if (counts[w] > std::numeric_limits<int64_t>::max() - t) return ACCO_ERR_ARG;
        t += counts[w];
    }
    *out = t;
    return ACCO_OK;
}

// Scalars of update number t = step + 1 on a gradient sum of total_count micro-batches.
AdamScalars fold(const acco_adamw_t& hp, int64_t step, int64_t total_count)
{
    const double t   = (double)(step + 1);
    const double bc1 = 1.0 - std::pow(hp.beta1, t);
    const double bc2 = 1.0 - std::pow(hp.beta2, t);
    AdamScalars  s;
    s.grad_scale = (float)(1.0 / (double)total_count);
    s.beta1      = (float)hp.beta1;
    s.beta2      = (float)hp.beta2;
    s.omb1       = (float)(1.0 - hp.beta1);
    s.omb2       = (float)(1.0 - hp.beta2);
    s.step_size  = (float)(hp.lr / bc1);
    s.rsqrt_bc2  = (float)(1.0 / std::sqrt(bc2));
    s.lrwd       = (float)(hp.lr * hp.weight_decay);
    s.eps        = (float)hp.eps;
    return s;
}

// ------------------------------------------------------------------ state layout

struct StateLayout {
    bool    blocked = false;
    int     vshift  = 0;   // log2(vectors per block)
    int64_t block   = 0;   // elements per block
    int64_t stride  = 0;   // elements between block starts
};

int parse_layout(const acco_layout_t* l, StateLayout* out)
{
    *out = StateLayout{};
    if (l == nullptr || l->block_elems == 0) return ACCO_OK;
    const int64_t b = l->block_elems, st = l->block_stride;
    if (b < 4 || b > ((int64_t)1 << 30) || (b & (b - 1)) != 0) return ACCO_ERR_ARG;
    if (st < b || st % 4 != 0 || st > ((int64_t)1 << 40)) return ACCO_ERR_ARG;
    out->blocked = true;
    out->block   = b;
    out->stride  = st;
    int sh       = 0;
    while (((int64_t)4 << sh) < b) ++sh;
    out->vshift = sh;
    return ACCO_OK;
}

// bytes from the first to one past the last element of an array of n elements of esz bytes
int64_t state_extent(const StateLayout& L, int64_t n, int64_t esz = 4)
{
    if (n <= 0) return 0;
    if (!L.blocked) return n * esz;
    const int64_t nblk = (n + L.block - 1) / L.block;
    return ((nblk - 1) * L.stride + (n - (nblk - 1) * L.block)) * esz;
}

// do two arrays of the same layout and element size share an element?
bool state_overlap(const void* a, const void* b, const StateLayout& L, int64_t n, int64_t esz = 4)
{
    const int64_t ext = state_extent(L, n, esz);
    if (!overlap(a, ext, b, ext)) return false;
    if (!L.blocked) return true;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    const uint64_t  period = (uint64_t)L.stride * esz, blk = (uint64_t)L.block * esz;
    const uint64_t  dist   = (pa > pb ? pa - pb : pb - pa) % period;
    return dist < blk || period - dist < blk;
}

// a planar buffer against a laid-out array (conservative for blocked layouts: whole extent)
bool planar_overlaps_state(const void* p, int64_t bytes, const void* state, const StateLayout& L,
                           int64_t n, int64_t esz = 4)
{
    return overlap(p, bytes, state, state_extent(L, n, esz));
}

template <class F>
int with_layout(const StateLayout& L, F&& f)
{
    if (L.blocked) return f(StateAddr<true>{L.vshift, L.stride / 4});
    return f(StateAddr<false>{});
}

template <class At>
constexpr bool is_blocked = std::is_same<At, StateAddr<true>>::value;

}  // namespace

// ------------------------------------------------------------------ entry points

ACCO_API int acco_accumulate(float* acc, const uint16_t* grad_bf16, int64_t n, int init,
                             int64_t* count, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && (acc == nullptr || grad_bf16 == nullptr)) return ACCO_ERR_NULL;
    if (!aligned16(acc) || !aligned16(grad_bf16)) return ACCO_ERR_ALIGN;
    if (init != 0 && init != 1) return ACCO_ERR_ARG;
    if (count != nullptr && !init &&
        (*count < 0 || *count == std::numeric_limits<int64_t>::max()))
        return ACCO_ERR_ARG;
    if (overlap(acc, n * 4, grad_bf16, n * 2)) return ACCO_ERR_ALIAS;

    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t s = static_cast<hipStream_t>(stream);
        if (init)
            rc = launch(kAccumulate, AccumulateOp<true>{acc, grad_bf16}, n, s, false);
        else
            rc = launch(kAccumulate, AccumulateOp<false>{acc, grad_bf16}, n, s);
    }
    if (rc == ACCO_OK && count != nullptr) *count = init ? 1 : *count + 1;
    return rc;
}

ACCO_API int acco_accumulate_bf16(uint16_t* acc_bf16, const uint16_t* grad_bf16, int64_t n, int init,
                                  int64_t* count, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && (acc_bf16 == nullptr || grad_bf16 == nullptr)) return ACCO_ERR_NULL;
    if (!aligned16(acc_bf16) || !aligned16(grad_bf16)) return ACCO_ERR_ALIGN;
    if (init != 0 && init != 1) return ACCO_ERR_ARG;
    if (count != nullptr && !init &&
        (*count < 0 || *count == std::numeric_limits<int64_t>::max()))
        return ACCO_ERR_ARG;
    if (overlap(acc_bf16, n * 2, grad_bf16, n * 2)) return ACCO_ERR_ALIAS;

    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t s = static_cast<hipStream_t>(stream);
        // in place: every lane reads its own elements of the running sum before it writes them
        rc = init ? launch(kStash, StashOp<false>{acc_bf16, grad_bf16, {}}, n, s)
                  : launch(kSecond, SecondPublishOp<>{acc_bf16, acc_bf16, grad_bf16, {}}, n, s);
    }
    if (rc == ACCO_OK && count != nullptr) *count = init ? 1 : *count + 1;
    return rc;
}

ACCO_API int acco_cast_params(uint16_t* out_bf16, const float* src, int64_t n, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && (out_bf16 == nullptr || src == nullptr)) return ACCO_ERR_NULL;
    if (!aligned16(out_bf16) || !aligned16(src)) return ACCO_ERR_ALIGN;
    if (overlap(out_bf16, n * 2, src, n * 4)) return ACCO_ERR_ALIAS;
    if (n == 0) return ACCO_OK;
    return launch(kCast, CastOp<>{out_bf16, src, {}}, n, static_cast<hipStream_t>(stream));
}


ACCO_API int acco_accumulate_first(uint16_t* stash_bf16, const uint16_t* grad_bf16, int64_t n,
                                   int publish, int64_t* count, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (publish != 0 && publish != 1) return ACCO_ERR_ARG;
    if (n > 0 && (stash_bf16 == nullptr || grad_bf16 == nullptr)) return ACCO_ERR_NULL;
    if (!aligned16(stash_bf16) || !aligned16(grad_bf16)) return ACCO_ERR_ALIGN;
    if (overlap(stash_bf16, n * 2, grad_bf16, n * 2)) return ACCO_ERR_ALIAS;
    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t s = static_cast<hipStream_t>(stream);
        rc = publish ? launch(kStash, StashOp<true>{stash_bf16, grad_bf16, {}}, n, s)
                     : launch(kStash, StashOp<false>{stash_bf16, grad_bf16, {}}, n, s);
    }
    if (rc == ACCO_OK && count != nullptr) *count = 1;
    return rc;
}

ACCO_API int acco_accumulate_second(float* acc, uint16_t* comm_bf16, const uint16_t* stash_bf16,
                                    const uint16_t* grad_bf16, int64_t n, int64_t* count,
                                    void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && (acc == nullptr) == (comm_bf16 == nullptr)) return ACCO_ERR_NULL;  // one output
    if (n > 0 && (stash_bf16 == nullptr || grad_bf16 == nullptr)) return ACCO_ERR_NULL;
    if (!aligned16(acc) || !aligned16(comm_bf16) || !aligned16(stash_bf16) || !aligned16(grad_bf16))
        return ACCO_ERR_ALIGN;
    if (count != nullptr && *count != 1) return ACCO_ERR_ARG;
    const void* ins[2] = {stash_bf16, grad_bf16};
    for (const void* in : ins)
        if (overlap(acc, n * 4, in, n * 2) || overlap(comm_bf16, n * 2, in, n * 2))
            return ACCO_ERR_ALIAS;
    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t s = static_cast<hipStream_t>(stream);
        rc = acc != nullptr ? launch(kSecond, SecondOp{acc, stash_bf16, grad_bf16}, n, s, false)
                            : launch(kSecond, SecondPublishOp<>{comm_bf16, stash_bf16, grad_bf16, {}}, n, s);
    }
    if (rc == ACCO_OK && count != nullptr) *count = 2;
    return rc;
}

ACCO_API int acco_accumulate_batch(int op, int workers, float* const* acc,
                                   uint16_t* const* out_bf16, const uint16_t* const* stash_bf16,
                                   const uint16_t* const* grad_bf16, int64_t n, int64_t* counts,
                                   const acco_layout_t* out_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (workers < 1 || workers > ACCO_MAX_WORKERS) return ACCO_ERR_SIZE;
    if (op < ACCO_BATCH_ACCUMULATE_INIT || op > ACCO_BATCH_RUNNING_BF16) return ACCO_ERR_ARG;
    // which columns the operation uses, and which one it writes
    const bool uses_acc   = op == ACCO_BATCH_ACCUMULATE_INIT || op == ACCO_BATCH_ACCUMULATE ||
                          op == ACCO_BATCH_ACCUMULATE_PUBLISH || op == ACCO_BATCH_SECOND ||
                          op == ACCO_BATCH_PUBLISH;
    const bool uses_out   = !(op == ACCO_BATCH_ACCUMULATE_INIT || op == ACCO_BATCH_ACCUMULATE ||
                            op == ACCO_BATCH_SECOND);
    const bool uses_stash = op == ACCO_BATCH_SECOND || op == ACCO_BATCH_SECOND_PUBLISH;
    const bool uses_grad  = op != ACCO_BATCH_PUBLISH;
    const bool writes_acc = uses_acc && !uses_out;
    if ((uses_acc && acc == nullptr) || (uses_out && out_bf16 == nullptr) ||
        (uses_stash && stash_bf16 == nullptr) || (uses_grad && grad_bf16 == nullptr))
        return ACCO_ERR_NULL;
    StateLayout OL;
    if (int rc = parse_layout(out_layout, &OL)) return rc;
    // a blocked output: only where there is an output, not for the in-place running sum, and
    // in blocks that hold whole 8-element vectors
    if (OL.blocked && (!uses_out || op == ACCO_BATCH_RUNNING_BF16 || OL.block < 8))
        return ACCO_ERR_ARG;

    // every buffer of the call as a byte range; written ranges must not meet any other range
    struct Range {
        const void* p;
        int64_t     bytes;   // extent
        bool        written;
        bool        laid;    // follows out_layout
    };
    Range ranges[4 * ACCO_MAX_WORKERS];
    int   nr = 0;
    for (int w = 0; w < workers; ++w) {
        const void* cols[4]  = {uses_acc ? (const void*)acc[w] : nullptr,
                                uses_out ? (const void*)out_bf16[w] : nullptr,
                                uses_stash ? (const void*)stash_bf16[w] : nullptr,
                                uses_grad ? (const void*)grad_bf16[w] : nullptr};
        const bool  used[4]  = {uses_acc, uses_out, uses_stash, uses_grad};
        const bool  wr[4]    = {writes_acc, uses_out, false, false};
        const int64_t esz[4] = {4, 2, 2, 2};
        for (int k = 0; k < 4; ++k) {
            if (!used[k]) continue;
            if (n > 0 && cols[k] == nullptr) return ACCO_ERR_NULL;
            if (!aligned16(cols[k])) return ACCO_ERR_ALIGN;
            const bool laid = k == 1 && OL.blocked;
            ranges[nr++] = Range{cols[k], laid ? state_extent(OL, n, 2) : n * esz[k], wr[k], laid};
        }
    }
    for (int i = 0; i < nr; ++i)
        for (int j = i + 1; j < nr; ++j) {
            if (!ranges[i].written && !ranges[j].written) continue;
            const bool hit = (ranges[i].laid && ranges[j].laid)
                                 ? state_overlap(ranges[i].p, ranges[j].p, OL, n, 2)
                                 : overlap(ranges[i].p, ranges[i].bytes, ranges[j].p, ranges[j].bytes);
            if (hit) return ACCO_ERR_ALIAS;
        }
    const bool starts  = op == ACCO_BATCH_ACCUMULATE_INIT || op == ACCO_BATCH_FIRST ||
                        op == ACCO_BATCH_FIRST_PUBLISH;
    const bool seconds = op == ACCO_BATCH_SECOND || op == ACCO_BATCH_SECOND_PUBLISH;
    if (counts != nullptr && op != ACCO_BATCH_PUBLISH && !starts)
        for (int w = 0; w < workers; ++w) {
            if (seconds ? counts[w] != 1
                        : (counts[w] < 0 || counts[w] == std::numeric_limits<int64_t>::max()))
                return ACCO_ERR_ARG;
        }

    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t        s = static_cast<hipStream_t>(stream);
        void* const*       A = reinterpret_cast<void* const*>(acc);
        void* const*       O = reinterpret_cast<void* const*>(out_bf16);
        const void* const* R = reinterpret_cast<const void* const*>(acc);
        const void* const* S = reinterpret_cast<const void* const*>(stash_bf16);
        const void* const* G = reinterpret_cast<const void* const*>(grad_bf16);
        const int          W = workers;
        switch (op) {
            case ACCO_BATCH_ACCUMULATE_INIT:
                rc = launch_batch<AccumulateOp<true>>(kAccumulate, A, G, nullptr, W, n, s, {}, false);
                break;
            case ACCO_BATCH_ACCUMULATE:
                rc = launch_batch<AccumulateOp<false>>(kAccumulate, A, G, nullptr, W, n, s);
                break;
            case ACCO_BATCH_SECOND:
                rc = launch_batch<SecondOp>(kSecond, A, G, S, W, n, s, {}, false);
                break;
            case ACCO_BATCH_RUNNING_BF16:  // in place: each lane reads its elements first
                rc = launch_batch<SecondPublishOp<>>(kSecond, O, G, reinterpret_cast<const void* const*>(out_bf16), W, n, s);
                break;
            default:
                // the operations with an output that may be laid out in blocks
                rc = with_layout(OL, [&](auto oat) {
                    constexpr bool B = is_blocked<decltype(oat)>;
                    switch (op) {
                        case ACCO_BATCH_ACCUMULATE_PUBLISH:
                            return launch_batch<AccumulatePublishOp<false, false, B>>(kAccumulatePublish, O, G, R, W, n, s, oat);
                        case ACCO_BATCH_FIRST:
                            return launch_batch<StashOp<false, B>>(kStash, O, G, nullptr, W, n, s, oat);
                        case ACCO_BATCH_FIRST_PUBLISH:
                            return launch_batch<StashOp<true, B>>(kStash, O, G, nullptr, W, n, s, oat);
                        case ACCO_BATCH_SECOND_PUBLISH:
                            return launch_batch<SecondPublishOp<B>>(kSecond, O, G, S, W, n, s, oat);
                        default:  // ACCO_BATCH_PUBLISH
                            return launch_batch<CastOp<B>>(kCast, O, nullptr, R, W, n, s, oat);
                    }
                });
                break;
        }
    }
    if (rc == ACCO_OK && counts != nullptr && op != ACCO_BATCH_PUBLISH)
        for (int w = 0; w < workers; ++w) counts[w] = starts ? 1 : counts[w] + 1;
    return rc;
}

namespace {

template <int WMAX>
ShardPtrs<WMAX> chunk_ptrs(const void* const* shards, int begin, int end)
{
    ShardPtrs<WMAX> ptrs;
    std::memset(&ptrs, 0, sizeof ptrs);
    for (int w = begin; w < end; ++w) ptrs.p[w - begin] = shards[w];
    return ptrs;
}

// Shards taken per launch by entry e: 8, or 16 bf16 shards when there are more than 8 (each
// pass over fewer than all shards costs a round trip of gsum: 8 bytes per element).  The
// 16-shard kernels exist in the flat shape only; with another shape selected it stays at 8.
template <bool BF16>
int reduce_chunk(Entry e, int workers, int64_t n)
{
    return BF16 && workers > kReduceChunk && flat_applies(e, n) ? kReduceChunkWide : kReduceChunk;
}

// f(integral_constant<int, WMAX>) with the kernel width that holds `cnt` shards
template <bool BF16, class F>
int with_width(int cnt, F&& f)
{
    if constexpr (BF16) {
        if (cnt > kReduceChunk) return f(std::integral_constant<int, kReduceChunkWide>{});
    }
    return f(std::integral_constant<int, kReduceChunk>{});
}

// The shards' own layout: only bf16 shards (the communication buffers) may be blocked.
template <bool BF16, class F>
int with_shard_layout(const StateLayout& SL, F&& f)
{
    if constexpr (BF16) {
        if (SL.blocked) return f(StateAddr<true>{SL.vshift, SL.stride / 4});
    }
    return f(StateAddr<false>{});
}

// plain reduction of shards [0, workers) into gsum, 8 or 16 at a time
template <bool BF16>
int launch_reduce(float* gsum, const StateLayout& L, const StateLayout& SL,
                  const void* const* shards, int workers, int64_t n, bool accumulate,
                  hipStream_t stream)
{
    const int chunk = reduce_chunk<BF16>(kReduce, workers, n);
    for (int w0 = 0; w0 < workers; w0 += chunk) {
        const int  end = w0 + chunk < workers ? w0 + chunk : workers;
        const bool acc = accumulate || w0 > 0;
        const int  rc  = with_width<BF16>(end - w0, [&](auto width) {
            constexpr int WM   = decltype(width)::value;
            const auto    ptrs = chunk_ptrs<WM>(shards, w0, end);
            return with_layout(L, [&](auto at) {
                return with_shard_layout<BF16>(SL, [&](auto sat) {
                    constexpr bool B = is_blocked<decltype(at)>, S = is_blocked<decltype(sat)>;
                    if (acc)
                        return launch(kReduce, ReduceOp<WM, BF16, true, B, S>{gsum, ptrs, end - w0, at, sat}, n, stream);
                    return launch(kReduce, ReduceOp<WM, BF16, false, B, S>{gsum, ptrs, end - w0, at, sat}, n, stream);
                });
            });
        });
        if (rc != ACCO_OK) return rc;
    }
    return ACCO_OK;
}

// the shards' layout argument: blocked layouts are for bf16 shards, in blocks of whole vectors
int parse_shard_layout(const acco_layout_t* l, int dtype, StateLayout* out)
{
    if (int rc = parse_layout(l, out)) return rc;
    if (out->blocked && dtype != ACCO_BF16) return ACCO_ERR_ARG;
    return ACCO_OK;
}

// shards: non-NULL (n > 0), aligned, none overlapping the state arrays listed
int check_shards_vs_state(const void* const* shards, int workers, int dtype, int64_t n,
                          const void* const* state, int nstate, const StateLayout& L,
                          const StateLayout& SL)
{
    if (workers < 1 || workers > ACCO_MAX_WORKERS) return ACCO_ERR_SIZE;
    if (dtype != ACCO_BF16 && dtype != ACCO_F32) return ACCO_ERR_ARG;
    const int64_t esz = dtype == ACCO_BF16 ? 2 : 4;
    for (int w = 0; w < workers; ++w) {
        if (n > 0 && shards[w] == nullptr) return ACCO_ERR_NULL;
        if (!aligned16(shards[w])) return ACCO_ERR_ALIGN;
        for (int k = 0; k < nstate; ++k)
            if (planar_overlaps_state(shards[w], state_extent(SL, n, esz), state[k], L, n))
                return ACCO_ERR_ALIAS;
    }
    return ACCO_OK;
}

}  // namespace

ACCO_API int acco_reduce_shards(float* gsum, const void* const* shards, int workers, int dtype,
                                int64_t n, int accumulate, const int64_t* counts, int64_t* total,
                                const acco_layout_t* gsum_layout,
                                const acco_layout_t* shard_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (shards == nullptr || (n > 0 && gsum == nullptr)) return ACCO_ERR_NULL;
    if (accumulate != 0 && accumulate != 1) return ACCO_ERR_ARG;
    if ((counts == nullptr) != (total == nullptr)) return ACCO_ERR_NULL;
    if (!aligned16(gsum)) return ACCO_ERR_ALIGN;
    StateLayout L, SL;
    if (int rc = parse_layout(gsum_layout, &L)) return rc;
    if (int rc = parse_shard_layout(shard_layout, dtype, &SL)) return rc;
    const void* st[1] = {gsum};
    if (int rc = check_shards_vs_state(shards, workers, dtype, n, st, 1, L, SL)) return rc;
    int64_t new_total = 0;
    if (counts != nullptr)
        if (int rc = sum_counts(counts, workers, accumulate ? *total : 0, &new_total)) return rc;

    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t s = static_cast<hipStream_t>(stream);
        rc = dtype == ACCO_BF16 ? launch_reduce<true>(gsum, L, SL, shards, workers, n, accumulate, s)
                                : launch_reduce<false>(gsum, L, SL, shards, workers, n, accumulate, s);
    }
    if (rc == ACCO_OK && total != nullptr) *total = new_total;
    return rc;
}

namespace {

// validation shared by the four AdamW step entry points.  outs: planar outputs (may be NULL).
int check_step_buffers(const float* theta, const float* m, const float* v, const float* gsum,
                       const void* out_f32, const void* out_bf16, int64_t n, const StateLayout& L)
{
    if (n > 0 && (theta == nullptr || m == nullptr || v == nullptr || gsum == nullptr))
        return ACCO_ERR_NULL;
    if (!aligned16(theta) || !aligned16(m) || !aligned16(v) || !aligned16(gsum) ||
        !aligned16(out_f32) || !aligned16(out_bf16))
        return ACCO_ERR_ALIGN;
    const void* st[4] = {theta, m, v, gsum};
    for (int a = 0; a < 4; ++a) {
        for (int b = a + 1; b < 4; ++b)
            if (state_overlap(st[a], st[b], L, n)) return ACCO_ERR_ALIAS;
        if (planar_overlaps_state(out_f32, n * 4, st[a], L, n)) return ACCO_ERR_ALIAS;
        if (planar_overlaps_state(out_bf16, n * 2, st[a], L, n)) return ACCO_ERR_ALIAS;
    }
    if (overlap(out_f32, n * 4, out_bf16, n * 2)) return ACCO_ERR_ALIAS;
    return ACCO_OK;
}

}  // namespace

namespace {

template <class SC>
constexpr bool from_device = std::is_same<SC, ScalarsFromDevice>::value;

// The device-scalar forms exist for the outputs a recorded round uses: bf16 theta~ for the
// estimate (no fp32 copy).
template <class SC>
int launch_estimate(const float* theta, const float* m, const float* v, const float* gsum,
                    float* o32, uint16_t* o16, int64_t n, const StateLayout& L, const SC& sc,
                    hipStream_t s)
{
    return with_layout(L, [&](auto at) {
        constexpr bool B = is_blocked<decltype(at)>;
        if constexpr (from_device<SC>) {
            if (o32 != nullptr || o16 == nullptr) return (int)ACCO_ERR_ARG;
        } else {
            if (o32 != nullptr && o16 != nullptr)
                return launch(kEstimate, AdamOp<false, true, true, B, SC>{theta, m, v, gsum, nullptr, nullptr, nullptr, o32, o16, sc, at}, n, s);
            if (o32 != nullptr)
                return launch(kEstimate, AdamOp<false, true, false, B, SC>{theta, m, v, gsum, nullptr, nullptr, nullptr, o32, nullptr, sc, at}, n, s);
        }
        return launch(kEstimate, AdamOp<false, false, true, B, SC>{theta, m, v, gsum, nullptr, nullptr, nullptr, nullptr, o16, sc, at}, n, s);
    });
}

template <class SC>
int launch_commit(float* theta, float* m, float* v, const float* gsum, uint16_t* o16, int64_t n,
                  const StateLayout& L, const SC& sc, hipStream_t s)
{
    return with_layout(L, [&](auto at) {
        constexpr bool B = is_blocked<decltype(at)>;
        if (o16 != nullptr)
            return launch(kCommit, AdamOp<true, false, true, B, SC>{theta, m, v, gsum, theta, m, v, nullptr, o16, sc, at}, n, s);
        return launch(kCommit, AdamOp<true, false, false, B, SC>{theta, m, v, gsum, theta, m, v, nullptr, nullptr, sc, at}, n, s);
    });
}

// the scalar block of the *_dev entry points: device memory, 16-byte aligned, clear of every
// buffer the call writes (conservative for blocked arrays: their whole extent)
int check_scalars_dev(const acco_step_scalars_t* p, const void* const* written,
                      const int64_t* bytes, int count)
{
    if (p == nullptr) return ACCO_ERR_NULL;
    if (!aligned16(p)) return ACCO_ERR_ALIGN;
    for (int k = 0; k < count; ++k)
        if (overlap(p, (int64_t)sizeof *p, written[k], bytes[k])) return ACCO_ERR_ALIAS;
    return ACCO_OK;
}

static_assert(sizeof(AdamScalars) <= sizeof(acco_step_scalars_t), "scalar block too small");
static_assert(sizeof(acco_step_scalars_t) == kWordsPerBlock * 4, "scalar block size");
static_assert(sizeof(StagedBlocks) == ACCO_STAGE_BLOCKS_MAX * sizeof(acco_step_scalars_t),
              "staging argument size");

}  // namespace

ACCO_API int acco_fold_adamw(const acco_adamw_t* hp, int64_t step, int64_t total_count,
                             acco_step_scalars_t* out)
{
    if (out == nullptr) return ACCO_ERR_NULL;
    if (int rc = check_hyper(hp, step, total_count)) return rc;
    const AdamScalars sc = fold(*hp, step, total_count);
    std::memset(out, 0, sizeof *out);
    std::memcpy(out, &sc, sizeof sc);
    return ACCO_OK;
}

ACCO_API int acco_stage_scalars(acco_step_scalars_t* dst_dev, const acco_step_scalars_t* src_host,
                                int blocks, void* stream)
{
    if (dst_dev == nullptr || src_host == nullptr) return ACCO_ERR_NULL;
    if (blocks < 1 || blocks > ACCO_STAGE_BLOCKS_MAX) return ACCO_ERR_SIZE;
    if (!aligned16(dst_dev)) return ACCO_ERR_ALIGN;
    StagedBlocks arg;
    std::memset(&arg, 0, sizeof arg);
    std::memcpy(arg.word, src_host, (size_t)blocks * sizeof *src_host);
    hipLaunchKernelGGL(stage_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<uint32_t*>(dst_dev), arg, blocks * kWordsPerBlock);
    return hipGetLastError() == hipSuccess ? ACCO_OK : ACCO_ERR_DEVICE;
}

ACCO_API int acco_estimate_step(const float* theta, const float* m, const float* v,
                                const float* gsum, float* theta_tilde_f32,
                                uint16_t* theta_tilde_bf16, int64_t n, const acco_adamw_t* hp,
                                int64_t step, int64_t total_count,
                                const acco_layout_t* state_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && theta_tilde_f32 == nullptr && theta_tilde_bf16 == nullptr) return ACCO_ERR_NULL;
    StateLayout L;
    if (int rc = parse_layout(state_layout, &L)) return rc;
    if (int rc = check_step_buffers(theta, m, v, gsum, theta_tilde_f32, theta_tilde_bf16, n, L))
        return rc;
    if (int rc = check_hyper(hp, step, total_count)) return rc;
    if (n == 0) return ACCO_OK;
    return launch_estimate(theta, m, v, gsum, theta_tilde_f32, theta_tilde_bf16, n, L,
                           ScalarsByValue{fold(*hp, step, total_count)},
                           static_cast<hipStream_t>(stream));
}

ACCO_API int acco_estimate_step_dev(const float* theta, const float* m, const float* v,
                                    const float* gsum, uint16_t* theta_tilde_bf16, int64_t n,
                                    const acco_step_scalars_t* scalars_dev,
                                    const acco_layout_t* state_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && theta_tilde_bf16 == nullptr) return ACCO_ERR_NULL;
    StateLayout L;
    if (int rc = parse_layout(state_layout, &L)) return rc;
    if (int rc = check_step_buffers(theta, m, v, gsum, nullptr, theta_tilde_bf16, n, L)) return rc;
    const void* written[1] = {theta_tilde_bf16};
    const int64_t bytes[1] = {n * 2};
    if (int rc = check_scalars_dev(scalars_dev, written, bytes, 1)) return rc;
    if (n == 0) return ACCO_OK;
    return launch_estimate(theta, m, v, gsum, nullptr, theta_tilde_bf16, n, L,
                           ScalarsFromDevice{reinterpret_cast<const AdamScalars*>(scalars_dev)},
                           static_cast<hipStream_t>(stream));
}

ACCO_API int acco_commit_step(float* theta, float* m, float* v, const float* gsum,
                              uint16_t* theta_bf16, int64_t n, const acco_adamw_t* hp,
                              int64_t* step, int64_t total_count,
                              const acco_layout_t* state_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (step == nullptr) return ACCO_ERR_NULL;
    StateLayout L;
    if (int rc = parse_layout(state_layout, &L)) return rc;
    if (int rc = check_step_buffers(theta, m, v, gsum, nullptr, theta_bf16, n, L)) return rc;
    if (int rc = check_hyper(hp, *step, total_count)) return rc;

    int rc = ACCO_OK;
    if (n > 0)
        rc = launch_commit(theta, m, v, gsum, theta_bf16, n, L,
                           ScalarsByValue{fold(*hp, *step, total_count)},
                           static_cast<hipStream_t>(stream));
    if (rc == ACCO_OK) *step += 1;
    return rc;
}

ACCO_API int acco_commit_step_dev(float* theta, float* m, float* v, const float* gsum,
                                  uint16_t* theta_bf16, int64_t n,
                                  const acco_step_scalars_t* scalars_dev,
                                  const acco_layout_t* state_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    StateLayout L;
    if (int rc = parse_layout(state_layout, &L)) return rc;
    if (int rc = check_step_buffers(theta, m, v, gsum, nullptr, theta_bf16, n, L)) return rc;
    const void* written[4] = {theta, m, v, theta_bf16};
    const int64_t ext      = state_extent(L, n);
    const int64_t bytes[4] = {ext, ext, ext, n * 2};
    if (int rc = check_scalars_dev(scalars_dev, written, bytes, 4)) return rc;
    if (n == 0) return ACCO_OK;
    return launch_commit(theta, m, v, gsum, theta_bf16, n, L,
                         ScalarsFromDevice{reinterpret_cast<const AdamScalars*>(scalars_dev)},
                         static_cast<hipStream_t>(stream));
}

// ------------------------------------------------------------------ resident scalar blocks

// Scalar blocks held by the library itself, for the one entry point that takes no device block
// from its caller.  Each device has its own copy of the array at its own address; in host code
// the array's name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) uint32_t scratch[ACCO_RESIDENT_SLOTS * acco::kWordsPerBlock];

namespace {

std::atomic<uint32_t*> g_scratch_ptr[64];   // per device: where that device's copy lives

// device address of block `slot` on the current device (looked up once per device)
int resident_block(int slot, uint32_t** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return ACCO_ERR_DEVICE;
    }
    uint32_t* base = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (base == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return ACCO_ERR_DEVICE;
        }
        base = static_cast<uint32_t*>(p);
        g_scratch_ptr[dev].store(base, std::memory_order_release);
    }
    *out = base + (int64_t)slot * kWordsPerBlock;
    return ACCO_OK;
}

}  // namespace

ACCO_API int acco_commit_step_resident(float* theta, float* m, float* v, const float* gsum,
                                       uint16_t* theta_bf16, int64_t n,
                                       const acco_step_scalars_t* scalars_host, int slot,
                                       const acco_layout_t* state_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (scalars_host == nullptr) return ACCO_ERR_NULL;
    if (slot < 0 || slot >= ACCO_RESIDENT_SLOTS) return ACCO_ERR_SIZE;
    StateLayout L;
    if (int rc = parse_layout(state_layout, &L)) return rc;
    if (int rc = check_step_buffers(theta, m, v, gsum, nullptr, theta_bf16, n, L)) return rc;
    if (n == 0) return ACCO_OK;
    uint32_t* block = nullptr;
    if (int rc = resident_block(slot, &block)) return rc;
    hipStream_t  s = static_cast<hipStream_t>(stream);
    StagedBlocks arg;
    std::memset(&arg, 0, sizeof arg);
    std::memcpy(arg.word, scalars_host, sizeof *scalars_host);
    // every word of the block is rewritten, so nothing of an earlier call survives in it
    hipLaunchKernelGGL(stage_kernel, dim3(1), dim3(64), 0, s, block, arg, kWordsPerBlock);
    if (hipGetLastError() != hipSuccess) return ACCO_ERR_DEVICE;
    return launch_commit(theta, m, v, gsum, theta_bf16, n, L,
                         ScalarsFromDevice{reinterpret_cast<const AdamScalars*>(block)}, s);
}

ACCO_API int acco_accumulate_publish(float* acc, const uint16_t* grad_bf16, uint16_t* comm_bf16,
                                     int64_t n, int init, int keep_acc, int64_t* count,
                                     void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (init != 0 && init != 1) return ACCO_ERR_ARG;
    if (keep_acc != 0 && keep_acc != 1) return ACCO_ERR_ARG;
    const bool needs_acc = !init || keep_acc;
    if (n > 0 && (grad_bf16 == nullptr || comm_bf16 == nullptr || (needs_acc && acc == nullptr)))
        return ACCO_ERR_NULL;
    if (!aligned16(acc) || !aligned16(grad_bf16) || !aligned16(comm_bf16)) return ACCO_ERR_ALIGN;
    if (count != nullptr && !init &&
        (*count < 0 || *count == std::numeric_limits<int64_t>::max()))
        return ACCO_ERR_ARG;
    if (overlap(acc, n * 4, grad_bf16, n * 2) || overlap(comm_bf16, n * 2, grad_bf16, n * 2) ||
        overlap(comm_bf16, n * 2, acc, n * 4))
        return ACCO_ERR_ALIAS;

    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t s = static_cast<hipStream_t>(stream);
        if (init && keep_acc)
            rc = launch(kAccumulatePublish, AccumulatePublishOp<true, true>{acc, grad_bf16, comm_bf16, {}}, n, s, false);
        else if (init)
            rc = launch(kAccumulatePublish, AccumulatePublishOp<true, false>{acc, grad_bf16, comm_bf16, {}}, n, s, false);
        else if (keep_acc)
            rc = launch(kAccumulatePublish, AccumulatePublishOp<false, true>{acc, grad_bf16, comm_bf16, {}}, n, s);
        else
            rc = launch(kAccumulatePublish, AccumulatePublishOp<false, false>{acc, grad_bf16, comm_bf16, {}}, n, s);
    }
    if (rc == ACCO_OK && count != nullptr) *count = init ? 1 : *count + 1;
    return rc;
}

namespace {

// Fused reduce + step over the last (up to `chunk`) shards; leading chunks of a larger
// worker count go through the plain reduction first.  The device-scalar forms have the bf16
// output only.
template <bool BF16, class SC>
int launch_reduce_estimate(const float* theta, const float* m, const float* v, float* gsum,
                           const StateLayout& L, const StateLayout& SL,
                           const void* const* shards, int workers, float* o32, uint16_t* o16,
                           int64_t n, const SC& sc, hipStream_t s)
{
    if (from_device<SC> && (o32 != nullptr || o16 == nullptr)) return ACCO_ERR_ARG;
    const int chunk = reduce_chunk<BF16>(kReduceEstimate, workers, n);
    const int lead  = ((workers - 1) / chunk) * chunk;
    if (lead > 0)
        if (int rc = launch_reduce<BF16>(gsum, L, SL, shards, lead, n, false, s)) return rc;
    const int cnt = workers - lead;
    return with_width<BF16>(cnt, [&](auto width) {
        constexpr int WM   = decltype(width)::value;
        const auto    ptrs = chunk_ptrs<WM>(shards, lead, workers);
        return with_layout(L, [&](auto at) {
            return with_shard_layout<BF16>(SL, [&](auto sat) {
                constexpr bool B = is_blocked<decltype(at)>, S = is_blocked<decltype(sat)>;
                auto go = [&](auto acc_tag) {
                    constexpr bool ACC = decltype(acc_tag)::value;
                    if constexpr (!from_device<SC>) {
                        if (o32 != nullptr && o16 != nullptr)
                            return launch(kReduceEstimate, ReduceAdamOp<false, BF16, ACC, true, true, true, B, S, SC, WM>{theta, m, v, gsum, ptrs, cnt, nullptr, nullptr, nullptr, o32, o16, sc, at, sat}, n, s);
                        if (o32 != nullptr)
                            return launch(kReduceEstimate, ReduceAdamOp<false, BF16, ACC, true, true, false, B, S, SC, WM>{theta, m, v, gsum, ptrs, cnt, nullptr, nullptr, nullptr, o32, nullptr, sc, at, sat}, n, s);
                    }
                    return launch(kReduceEstimate, ReduceAdamOp<false, BF16, ACC, true, false, true, B, S, SC, WM>{theta, m, v, gsum, ptrs, cnt, nullptr, nullptr, nullptr, nullptr, o16, sc, at, sat}, n, s);
                };
                return lead > 0 ? go(std::true_type{}) : go(std::false_type{});
            });
        });
    });
}

template <bool BF16, class SC>
int launch_reduce_commit(float* theta, float* m, float* v, float* gsum, const StateLayout& L,
                         const StateLayout& SL, const void* const* shards, int workers,
                         uint16_t* o16, int64_t n, const SC& sc, hipStream_t s)
{
    const int chunk = reduce_chunk<BF16>(kReduceCommit, workers, n);
    const int lead  = ((workers - 1) / chunk) * chunk;
    if (lead > 0)
        if (int rc = launch_reduce<BF16>(gsum, L, SL, shards, lead, n, true, s)) return rc;
    const int cnt = workers - lead;
    return with_width<BF16>(cnt, [&](auto width) {
        constexpr int WM   = decltype(width)::value;
        const auto    ptrs = chunk_ptrs<WM>(shards, lead, workers);
        return with_layout(L, [&](auto at) {
            return with_shard_layout<BF16>(SL, [&](auto sat) {
                constexpr bool B = is_blocked<decltype(at)>, S = is_blocked<decltype(sat)>;
                if (o16 != nullptr)
                    return launch(kReduceCommit, ReduceAdamOp<true, BF16, true, false, false, true, B, S, SC, WM>{theta, m, v, gsum, ptrs, cnt, theta, m, v, nullptr, o16, sc, at, sat}, n, s);
                return launch(kReduceCommit, ReduceAdamOp<true, BF16, true, false, false, false, B, S, SC, WM>{theta, m, v, gsum, ptrs, cnt, theta, m, v, nullptr, nullptr, sc, at, sat}, n, s);
            });
        });
    });
}

// validation shared by the by-value and the device-scalar forms of the two fused entry points
int check_reduce_step(const float* theta, const float* m, const float* v, const float* gsum,
                      const void* const* shards, int workers, int dtype, const void* out_f32,
                      const void* out_bf16, int64_t n, const acco_layout_t* state_layout,
                      const acco_layout_t* shard_layout, StateLayout* L, StateLayout* SL)
{
    if (int rc = parse_layout(state_layout, L)) return rc;
    if (int rc = parse_shard_layout(shard_layout, dtype, SL)) return rc;
    if (int rc = check_step_buffers(theta, m, v, gsum, out_f32, out_bf16, n, *L)) return rc;
    const void* st[4] = {theta, m, v, gsum};
    if (int rc = check_shards_vs_state(shards, workers, dtype, n, st, 4, *L, *SL)) return rc;
    const int64_t ext = state_extent(*SL, n, dtype == ACCO_BF16 ? 2 : 4);
    for (int w = 0; w < workers; ++w)
        if (overlap(out_f32, n * 4, shards[w], ext) || overlap(out_bf16, n * 2, shards[w], ext))
            return ACCO_ERR_ALIAS;
    return ACCO_OK;
}

}  // namespace

ACCO_API int acco_reduce_estimate_step(const float* theta, const float* m, const float* v,
                                       float* gsum, const void* const* shards, int workers,
                                       int dtype, const int64_t* counts, int64_t* total,
                                       float* theta_tilde_f32, uint16_t* theta_tilde_bf16,
                                       int64_t n, const acco_adamw_t* hp, int64_t step,
                                       const acco_layout_t* state_layout,
                                       const acco_layout_t* shard_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (shards == nullptr || counts == nullptr || total == nullptr) return ACCO_ERR_NULL;
    if (n > 0 && theta_tilde_f32 == nullptr && theta_tilde_bf16 == nullptr) return ACCO_ERR_NULL;
    StateLayout L, SL;
    if (int rc = check_reduce_step(theta, m, v, gsum, shards, workers, dtype, theta_tilde_f32,
                                   theta_tilde_bf16, n, state_layout, shard_layout, &L, &SL))
        return rc;
    int64_t new_total = 0;
    if (int rc = sum_counts(counts, workers, 0, &new_total)) return rc;
    if (int rc = check_hyper(hp, step, new_total)) return rc;

    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t          s  = static_cast<hipStream_t>(stream);
        const ScalarsByValue sc = {fold(*hp, step, new_total)};
        rc = dtype == ACCO_BF16
                 ? launch_reduce_estimate<true>(theta, m, v, gsum, L, SL, shards, workers, theta_tilde_f32, theta_tilde_bf16, n, sc, s)
                 : launch_reduce_estimate<false>(theta, m, v, gsum, L, SL, shards, workers, theta_tilde_f32, theta_tilde_bf16, n, sc, s);
    }
    if (rc == ACCO_OK) *total = new_total;
    return rc;
}

ACCO_API int acco_reduce_estimate_step_dev(const float* theta, const float* m, const float* v,
                                           float* gsum, const void* const* shards, int workers,
                                           int dtype, uint16_t* theta_tilde_bf16, int64_t n,
                                           const acco_step_scalars_t* scalars_dev,
                                           const acco_layout_t* state_layout,
                                           const acco_layout_t* shard_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (shards == nullptr || (n > 0 && theta_tilde_bf16 == nullptr)) return ACCO_ERR_NULL;
    StateLayout L, SL;
    if (int rc = check_reduce_step(theta, m, v, gsum, shards, workers, dtype, nullptr,
                                   theta_tilde_bf16, n, state_layout, shard_layout, &L, &SL))
        return rc;
    const void* written[2] = {gsum, theta_tilde_bf16};
    const int64_t bytes[2] = {state_extent(L, n), n * 2};
    if (int rc = check_scalars_dev(scalars_dev, written, bytes, 2)) return rc;
    if (n == 0) return ACCO_OK;
    hipStream_t             s  = static_cast<hipStream_t>(stream);
    const ScalarsFromDevice sc = {reinterpret_cast<const AdamScalars*>(scalars_dev)};
    return dtype == ACCO_BF16
               ? launch_reduce_estimate<true>(theta, m, v, gsum, L, SL, shards, workers, nullptr, theta_tilde_bf16, n, sc, s)
               : launch_reduce_estimate<false>(theta, m, v, gsum, L, SL, shards, workers, nullptr, theta_tilde_bf16, n, sc, s);
}

ACCO_API int acco_reduce_commit_step(float* theta, float* m, float* v, float* gsum,
                                     const void* const* shards, int workers, int dtype,
                                     const int64_t* counts, int64_t* total, uint16_t* theta_bf16,
                                     int64_t n, const acco_adamw_t* hp, int64_t* step,
                                     const acco_layout_t* state_layout,
                                     const acco_layout_t* shard_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (shards == nullptr || counts == nullptr || total == nullptr || step == nullptr)
        return ACCO_ERR_NULL;
    StateLayout L, SL;
    if (int rc = check_reduce_step(theta, m, v, gsum, shards, workers, dtype, nullptr, theta_bf16,
                                   n, state_layout, shard_layout, &L, &SL))
        return rc;
    int64_t new_total = 0;
    if (int rc = sum_counts(counts, workers, *total, &new_total)) return rc;
    if (int rc = check_hyper(hp, *step, new_total)) return rc;

    int rc = ACCO_OK;
    if (n > 0) {
        hipStream_t          s  = static_cast<hipStream_t>(stream);
        const ScalarsByValue sc = {fold(*hp, *step, new_total)};
        rc = dtype == ACCO_BF16
                 ? launch_reduce_commit<true>(theta, m, v, gsum, L, SL, shards, workers, theta_bf16, n, sc, s)
                 : launch_reduce_commit<false>(theta, m, v, gsum, L, SL, shards, workers, theta_bf16, n, sc, s);
    }
    if (rc == ACCO_OK) {
        *total = new_total;
        *step += 1;
    }
    return rc;
}

ACCO_API int acco_reduce_commit_step_dev(float* theta, float* m, float* v, float* gsum,
                                         const void* const* shards, int workers, int dtype,
                                         uint16_t* theta_bf16, int64_t n,
                                         const acco_step_scalars_t* scalars_dev,
                                         const acco_layout_t* state_layout,
                                         const acco_layout_t* shard_layout, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (shards == nullptr) return ACCO_ERR_NULL;
    StateLayout L, SL;
    if (int rc = check_reduce_step(theta, m, v, gsum, shards, workers, dtype, nullptr, theta_bf16,
                                   n, state_layout, shard_layout, &L, &SL))
        return rc;
    const void* written[5] = {theta, m, v, gsum, theta_bf16};
    const int64_t ext      = state_extent(L, n);
    const int64_t bytes[5] = {ext, ext, ext, ext, n * 2};
    if (int rc = check_scalars_dev(scalars_dev, written, bytes, 5)) return rc;
    if (n == 0) return ACCO_OK;
    hipStream_t             s  = static_cast<hipStream_t>(stream);
    const ScalarsFromDevice sc = {reinterpret_cast<const AdamScalars*>(scalars_dev)};
    return dtype == ACCO_BF16
               ? launch_reduce_commit<true>(theta, m, v, gsum, L, SL, shards, workers, theta_bf16, n, sc, s)
               : launch_reduce_commit<false>(theta, m, v, gsum, L, SL, shards, workers, theta_bf16, n, sc, s);
}

namespace {

int check_sgd(const acco_sgd_t* hp, int64_t total_count)
{
    if (hp == nullptr) return ACCO_ERR_NULL;
    if (!finite_nonneg(hp->lr) || !finite_nonneg(hp->weight_decay) || total_count < 1)
        return ACCO_ERR_ARG;
    return ACCO_OK;
}

SgdScalars fold_sgd(const acco_sgd_t& hp, int64_t total_count)
{
    SgdScalars s;
    s.grad_scale = (float)(1.0 / (double)total_count);
    s.lr         = (float)hp.lr;
    s.lrwd       = (float)(hp.lr * hp.weight_decay);
    return s;
}

}  // namespace

ACCO_API int acco_sgd_estimate_step(const float* theta, const float* gsum, float* theta_tilde_f32,
                                    uint16_t* theta_tilde_bf16, int64_t n, const acco_sgd_t* hp,
                                    int64_t total_count, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && (theta == nullptr || gsum == nullptr)) return ACCO_ERR_NULL;
    if (n > 0 && theta_tilde_f32 == nullptr && theta_tilde_bf16 == nullptr) return ACCO_ERR_NULL;
    if (!aligned16(theta) || !aligned16(gsum) || !aligned16(theta_tilde_f32) ||
        !aligned16(theta_tilde_bf16))
        return ACCO_ERR_ALIGN;
    if (int rc = check_sgd(hp, total_count)) return rc;
    const void* ins[2] = {theta, gsum};
    for (const void* in : ins) {
        if (overlap(theta_tilde_f32, n * 4, in, n * 4)) return ACCO_ERR_ALIAS;
        if (overlap(theta_tilde_bf16, n * 2, in, n * 4)) return ACCO_ERR_ALIAS;
    }
    if (overlap(theta_tilde_f32, n * 4, theta_tilde_bf16, n * 2)) return ACCO_ERR_ALIAS;
    if (n == 0) return ACCO_OK;
    const SgdScalars sc = fold_sgd(*hp, total_count);
    hipStream_t      s  = static_cast<hipStream_t>(stream);
    if (theta_tilde_f32 != nullptr && theta_tilde_bf16 != nullptr)
        return launch(kSgd, SgdOp<false, true, true>{theta, gsum, nullptr, theta_tilde_f32, theta_tilde_bf16, sc}, n, s);
    if (theta_tilde_f32 != nullptr)
        return launch(kSgd, SgdOp<false, true, false>{theta, gsum, nullptr, theta_tilde_f32, nullptr, sc}, n, s);
    return launch(kSgd, SgdOp<false, false, true>{theta, gsum, nullptr, nullptr, theta_tilde_bf16, sc}, n, s);
}

ACCO_API int acco_sgd_commit_step(float* theta, const float* gsum, uint16_t* theta_bf16, int64_t n,
                                  const acco_sgd_t* hp, int64_t* step, int64_t total_count,
                                  void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (step == nullptr) return ACCO_ERR_NULL;
    if (n > 0 && (theta == nullptr || gsum == nullptr)) return ACCO_ERR_NULL;
    if (!aligned16(theta) || !aligned16(gsum) || !aligned16(theta_bf16)) return ACCO_ERR_ALIGN;
    if (int rc = check_sgd(hp, total_count)) return rc;
    if (*step < 0 || *step == std::numeric_limits<int64_t>::max()) return ACCO_ERR_ARG;
    if (overlap(theta, n * 4, gsum, n * 4) || overlap(theta_bf16, n * 2, theta, n * 4) ||
        overlap(theta_bf16, n * 2, gsum, n * 4))
        return ACCO_ERR_ALIAS;
    int rc = ACCO_OK;
    if (n > 0) {
        const SgdScalars sc = fold_sgd(*hp, total_count);
        hipStream_t      s  = static_cast<hipStream_t>(stream);
        if (theta_bf16 != nullptr)
            rc = launch(kSgd, SgdOp<true, false, true>{theta, gsum, theta, nullptr, theta_bf16, sc}, n, s);
        else
            rc = launch(kSgd, SgdOp<true, false, false>{theta, gsum, theta, nullptr, nullptr, sc}, n, s);
    }
    if (rc == ACCO_OK) *step += 1;
    return rc;
}

ACCO_API int acco_probe_copy(float* dst, const float* src, int64_t n, void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && (dst == nullptr || src == nullptr)) return ACCO_ERR_NULL;
    if (!aligned16(dst) || !aligned16(src)) return ACCO_ERR_ALIGN;
    if (overlap(dst, n * 4, src, n * 4)) return ACCO_ERR_ALIAS;
    if (n == 0) return ACCO_OK;
    return launch(kProbe, ProbeCopyOp{dst, src}, n, static_cast<hipStream_t>(stream));
}

ACCO_API int acco_probe_triad(float* a, float* b, float* c, const float* d, int64_t n,
                              void* stream)
{
    if (int rc = check_n(n)) return rc;
    if (n > 0 && (a == nullptr || b == nullptr || c == nullptr || d == nullptr))
        return ACCO_ERR_NULL;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c) || !aligned16(d)) return ACCO_ERR_ALIGN;
    const void* arr[4] = {a, b, c, d};
    for (int i = 0; i < 4; ++i)
        for (int j = i + 1; j < 4; ++j)
            if (overlap(arr[i], n * 4, arr[j], n * 4)) return ACCO_ERR_ALIAS;
    if (n == 0) return ACCO_OK;
    return launch(kProbe, ProbeTriadOp{a, b, c, d}, n, static_cast<hipStream_t>(stream));
}

// ------------------------------------------------------------------ memory classes

namespace {

struct PairTimer {
    hipEvent_t  e0 = nullptr, e1 = nullptr;
    hipStream_t stream;
    uint32_t*   out;
    int64_t     words;
    bool        ok = true;

    PairTimer(hipStream_t s, uint32_t* o, int64_t w) : stream(s), out(o), words(w)
    {
        ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
    }
    ~PairTimer()
    {
        if (e0 != nullptr) (void)hipEventDestroy(e0);
        if (e1 != nullptr) (void)hipEventDestroy(e1);
    }
    // fastest of `reps` timed launches reading at a and b (ms); < 0 on a runtime error
    float time(const uint32_t* a, const uint32_t* b, int reps)
    {
        float best = -1.0f;
        for (int r = 0; r <= reps && ok; ++r) {   // launch 0 is a warm-up
            ok = ok && hipEventRecord(e0, stream) == hipSuccess;
            ok = ok && launch(kSecond, ProbePairOp{out, a, b}, words, stream) == ACCO_OK;
            ok = ok && hipEventRecord(e1, stream) == hipSuccess;
            ok = ok && hipEventSynchronize(e1) == hipSuccess;
            float ms = 0.0f;
            ok       = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
            if (ok && r > 0 && (best < 0.0f || ms < best)) best = ms;
        }
        return ok ? best : -1.0f;
    }
};

constexpr float kSlowPair = 1.045f;   // the two populations measured 8-10 % apart on MI355X

}  // namespace

ACCO_API int acco_hbm_classify(const void* base, int64_t bytes, int64_t step_bytes,
                               int64_t probe_bytes, void* scratch, int32_t* classes,
                               int64_t count, int32_t* n_classes, void* stream)
{
    if (base == nullptr || scratch == nullptr || classes == nullptr || n_classes == nullptr)
        return ACCO_ERR_NULL;
    if (!aligned16(base) || !aligned16(scratch)) return ACCO_ERR_ALIGN;
    if (probe_bytes < 4096 || probe_bytes % 4096 != 0 || probe_bytes > ((int64_t)1 << 34) ||
        step_bytes < 4096 || step_bytes % 4096 != 0 || bytes < probe_bytes)
        return ACCO_ERR_SIZE;
    if (count != (bytes - probe_bytes) / step_bytes + 1 || count > ((int64_t)1 << 20))
        return ACCO_ERR_SIZE;
    if (overlap(base, bytes, scratch, probe_bytes)) return ACCO_ERR_ALIAS;

    const char* p0 = static_cast<const char*>(base);
    auto        at = [&](int64_t k) { return reinterpret_cast<const uint32_t*>(p0 + k * step_bytes); };
    PairTimer   timer(static_cast<hipStream_t>(stream), static_cast<uint32_t*>(scratch),
                      probe_bytes / 4);
    if (!timer.ok) return ACCO_ERR_DEVICE;
    for (int64_t k = 0; k < count; ++k) classes[k] = -1;
    if (count == 1) {
        classes[0] = 0;
        *n_classes = 1;
        return ACCO_OK;
    }
    // what a pair in ONE class takes: the fastest of some pairs of neighbouring positions
    // (classes are tens of GiB long, so nearly all neighbours share one; disturbances only
    // ever add time)
    float   cal[12];
    int     ncal = 0;
    const int64_t stride = count > 24 ? (count - 1) / 12 : 1;
    for (int64_t k = 0; k + 1 < count && ncal < 12; k += stride) {
        const float t = timer.time(at(k), at(k + 1), 3);
        if (t < 0.0f) return ACCO_ERR_DEVICE;
        cal[ncal++] = t;
    }
    const float fast = *std::min_element(cal, cal + ncal);

    // first fit against one reference position per class found so far
    int64_t refs[64];
    int     nref = 0;
    for (int64_t k = 0; k < count; ++k) {
        int found = -1;
        // a disturbance can only make a pair look slow, never fast: a position that matches no
        // class gets a second round of probes before it founds a new one
        for (int attempt = 0; attempt < 2 && found < 0; ++attempt)
            for (int c = 0; c < nref && found < 0; ++c) {
                const float t = timer.time(at(refs[c]), at(k), 3);
                if (t < 0.0f) return ACCO_ERR_DEVICE;
                if (t < fast * kSlowPair) found = c;
            }
        if (found < 0) {
            if (nref == 64) return ACCO_ERR_DEVICE;   // timings too erratic to classify
            refs[nref] = k;
            found      = nref++;
        }
        classes[k] = found;
    }
    // a lone position between two neighbours of one class is a timing hiccup
    for (int64_t k = 1; k + 1 < count; ++k)
        if (classes[k - 1] == classes[k + 1] && classes[k] != classes[k - 1]) classes[k] = classes[k - 1];
    // number the classes by size, largest first
    int64_t size[64] = {0};
    int     order[64], rank[64];
    for (int64_t k = 0; k < count; ++k) size[classes[k]] += 1;
    for (int c = 0; c < nref; ++c) order[c] = c;
    for (int i = 1; i < nref; ++i)
        for (int j = i; j > 0 && size[order[j]] > size[order[j - 1]]; --j) std::swap(order[j], order[j - 1]);
    int used = 0;
    for (int i = 0; i < nref; ++i) {
        rank[order[i]] = i;
        if (size[order[i]] > 0) used = i + 1;
    }
    for (int64_t k = 0; k < count; ++k) classes[k] = rank[classes[k]];
    *n_classes = used;
    return ACCO_OK;
}

ACCO_API double acco_lr_cosine(double base_lr, double min_lr, int64_t step, int64_t warmup_steps,
                               int64_t total_steps)
{
    const double nan = std::numeric_limits<double>::quiet_NaN();
    if (!finite_nonneg(base_lr) || !finite_nonneg(min_lr) || min_lr > base_lr) return nan;
    if (step < 0 || warmup_steps < 0 || total_steps < warmup_steps) return nan;
    if (step < warmup_steps) return base_lr * (double)(step + 1) / (double)warmup_steps;
    const int64_t span = total_steps - warmup_steps;
    double        p    = (double)(step - warmup_steps) / (double)(span > 0 ? span : 1);
    if (p > 1.0) p = 1.0;
    const double pi = 3.14159265358979323846;
    return min_lr + (base_lr - min_lr) * (1.0 + std::cos(pi * p)) * 0.5;
}

ACCO_API const char* acco_status_string(int status)
{
    switch (status) {
        case ACCO_OK: return "ACCO_OK";
        case ACCO_ERR_NULL: return "ACCO_ERR_NULL: a required pointer is NULL";
        case ACCO_ERR_SIZE: return "ACCO_ERR_SIZE: element, worker, block or slot count out of range";
        case ACCO_ERR_ALIGN: return "ACCO_ERR_ALIGN: device pointer not 16-byte aligned";
        case ACCO_ERR_ARG: return "ACCO_ERR_ARG: invalid hyper-parameter, count, step, dtype or flag";
        case ACCO_ERR_ALIAS: return "ACCO_ERR_ALIAS: output overlaps an input";
        case ACCO_ERR_DEVICE: return "ACCO_ERR_DEVICE: HIP runtime error at launch";
        default: return "ACCO: unknown status";
    }
}

ACCO_API int acco_version(void)
{
    return 500;  // 0.5.0
}

ACCO_API void acco_reset_launch_settings(void)
{
    reset_shapes();
}

ACCO_API int acco_set_resident_waves(const char* entry, int waves_per_cu)
{
    if (entry == nullptr) return ACCO_ERR_NULL;
    // at least 3 workgroups must fit: one workgroup may reserve at most 64 KiB of LDS
    if (waves_per_cu != 0 && (waves_per_cu < 3 || waves_per_cu > 32)) return ACCO_ERR_ARG;
    for (int e = 0; e < kEntries; ++e) {
        if (std::strcmp(entry, kEntryNames[e]) == 0) {
            uint64_t old = g_shape[e].load(std::memory_order_relaxed);
            for (;;) {
                LaunchShape sh = unpack_shape(old);
                if (waves_per_cu != 0 && waves_per_cu / (sh.threads / 64) < 3) return ACCO_ERR_ARG;
                sh.resident = waves_per_cu;
                if (g_shape[e].compare_exchange_weak(old, pack_shape(sh), std::memory_order_relaxed))
                    return ACCO_OK;
            }
        }
    }
    return ACCO_ERR_ARG;
}

ACCO_API int acco_set_launch_shape(const char* entry, int threads, int vectors_in_flight,
                                   int workgroups_per_cu)
{
    if (entry == nullptr) return ACCO_ERR_NULL;
    if (threads < 64 || threads > kMaxThreads || threads % 64 != 0) return ACCO_ERR_ARG;
    if (vectors_in_flight != 1 && vectors_in_flight != 2 && vectors_in_flight != 4)
        return ACCO_ERR_ARG;
    if (workgroups_per_cu < 0 || workgroups_per_cu > 64) return ACCO_ERR_ARG;
    for (int e = 0; e < kEntries; ++e) {
        if (std::strcmp(entry, kEntryNames[e]) == 0) {
            uint64_t old = g_shape[e].load(std::memory_order_relaxed);
            for (;;) {
                LaunchShape sh = unpack_shape(old);
                sh.threads     = threads;
                sh.vectors     = vectors_in_flight;
                sh.wg_per_cu   = workgroups_per_cu;
                if (g_shape[e].compare_exchange_weak(old, pack_shape(sh), std::memory_order_relaxed))
                    return ACCO_OK;
            }
        }
    }
    return ACCO_ERR_ARG;
}
