// Device code of the ACCO shard path for gfx950: streaming kernels, all elementwise
// and HBM-bound (no MFMA, nothing staged in LDS), each built from an "Op" (what to load, what to
// compute, what to store for one vector) and one of two drivers.
//
// A "vector" is 4 consecutive elements: 16 bytes of fp32 (one dwordx4 per lane) or
// 8 bytes of bf16 (one dwordx2 per lane), so each wavefront instruction touches 1024
// (512) contiguous bytes.  Kernels whose arrays are all bf16 take 8 elements (one
// dwordx4) per lane instead.
//   flat_kernel    one vector per thread, one tile per workgroup, no loop: the default;
//   stream_kernel  grid-stride over tiles of T*U vectors, the loads of a thread's U
//                  vectors of every input issued before the first use (kept selectable
//                  through acco_set_launch_shape; slower at every size measured).
// The elements after the last whole vector are done one by one by workgroup 0.
// Both drivers take the Op from a "source": Single<Op> holds one Op; Batch<Op> holds a table
// of pointers for up to kBatchMax workers and builds the Op of worker blockIdx.y from it, so
// that the same accumulation step of several workers runs as ONE launch (grid.y = workers).
//
// Arithmetic: fp32, one IEEE operation per written operation (compiled with
// -ffp-contract=off; the fused multiply-adds below are explicit), correctly
// rounded division and square root, denormals kept.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace acco {

typedef float    f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

constexpr int kReduceChunk     = 8;   // worker shards summed per launch
constexpr int kReduceChunkWide = 16;  // the same for bf16 shards when there are more than 8
constexpr int kBatchMax    = 16;  // workers' accumulations served by one batched launch
constexpr int kMaxThreads = 512;  // per workgroup: leaves 256 VGPRs per lane for loads in flight

// ------------------------------------------------------------------ state addressing

// Where element j of a state array (theta, m, v, gsum) lives.  Planar: at index j.
// Blocked: the array is cut into blocks of 2^k elements whose starts are `stride`
// elements apart, so that theta, m, v and gsum of the same elements can sit next to
// each other in one buffer ([theta block][m block][v block][gsum block] ...), which
// keeps the concurrently streamed addresses within a few tens of KiB of each other.
template <bool BLOCKED>
struct StateAddr;

template <>
struct StateAddr<false> {
    __device__ __forceinline__ int64_t vec(int64_t i) const { return i; }
    __device__ __forceinline__ int64_t elem(int64_t j) const { return j; }
};

template <>
struct StateAddr<true> {
    int     vshift;   // log2(vectors per block)
    int64_t vstride;  // vectors between block starts
    __device__ __forceinline__ int64_t vec(int64_t i) const
    {
        return (i >> vshift) * vstride + (i & (((int64_t)1 << vshift) - 1));
    }
    __device__ __forceinline__ int64_t elem(int64_t j) const
    {
        return (j >> (vshift + 2)) * (vstride * 4) + (j & (((int64_t)4 << vshift) - 1));
    }
};

// ------------------------------------------------------------------ bf16 <-> fp32

__device__ __forceinline__ float bf16_lo(uint32_t packed)
{
    return __uint_as_float(packed << 16);
}

__device__ __forceinline__ float bf16_hi(uint32_t packed)
{
    return __uint_as_float(packed & 0xFFFF0000u);
}

// round to nearest even on the upper half; NaN keeps its sign and gets the quiet bit
__device__ __forceinline__ uint32_t to_bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    uint32_t r = u + 0x7FFFu + ((u >> 16) & 1u);
    r          = ((u & 0x7FFFFFFFu) > 0x7F800000u) ? (u | 0x00400000u) : r;
    return r >> 16;
}

__device__ __forceinline__ u2 pack_bf16x4(f4 x)
{
    u2 p;
    p.x = to_bf16_bits(x.x) | (to_bf16_bits(x.y) << 16);
    p.y = to_bf16_bits(x.z) | (to_bf16_bits(x.w) << 16);
    return p;
}

__device__ __forceinline__ f4 unpack_bf16x4(u2 p)
{
    f4 x;
    x.x = bf16_lo(p.x);
    x.y = bf16_hi(p.x);
    x.z = bf16_lo(p.y);
    x.w = bf16_hi(p.y);
    return x;
}

// ------------------------------------------------------------------ AdamW element update

// Host-folded scalars of one update (computed in double, rounded once).
struct AdamScalars {
    float grad_scale;  // 1 / total micro-batch count
    float beta1, beta2;
    float omb1, omb2;  // 1 - beta
    float step_size;   // lr / (1 - beta1^t)
    float rsqrt_bc2;   // 1 / sqrt(1 - beta2^t)
    float lrwd;        // lr * weight_decay
    float eps;
};

// Where a step kernel takes its scalars from: the kernel arguments (the usual case), or a block
// in device memory that is read when the kernel RUNS - a launch recorded into a graph then
// follows the scalars the host stages there before each replay (the update index, and with it
// the bias corrections, change every round).
struct ScalarsByValue {
    AdamScalars s;
    __device__ __forceinline__ const AdamScalars& get() const { return s; }
};

struct ScalarsFromDevice {
    const AdamScalars* p;
    __device__ __forceinline__ AdamScalars get() const { return *p; }
};

// Puts scalar blocks that travel in the kernel arguments into device memory (one wavefront;
// 16 words per block).  Kernels later on the same stream read them there.
constexpr int kWordsPerBlock   = 16;
constexpr int kStagedWordsMax  = 64;

struct StagedBlocks {
    uint32_t word[kStagedWordsMax];
};

__global__ void __launch_bounds__(64) stage_kernel(uint32_t* dst, const StagedBlocks src,
                                                   const int words)
{
    // lane i picks word i by a chain of selects: the argument words stay in scalar registers
    // (indexing them by lane would spill the whole block to private memory)
    const int i = (int)threadIdx.x;
    uint32_t  x = 0;
#pragma unroll
    for (int k = 0; k < kStagedWordsMax; ++k) x = (i == k) ? src.word[k] : x;
    if (i < words) dst[i] = x;
}

// AdamW with decoupled decay on theta(t), bias-corrected moments, eps added to the
// bias-corrected root.  `/` and __builtin_sqrtf compile to the correctly rounded
// sequences (the __fsqrt_rn intrinsic does not: it was measured 1 ulp off on gfx950).
// The decay is theta - (lr wd) theta in one fused operation (a pre-rounded factor
// 1 - lr wd would bias theta on every step).
__device__ __forceinline__ void adamw_elem(float theta, float m, float v, float gsum,
                                           const AdamScalars& s, float& theta_o, float& m_o,
                                           float& v_o)
{
    const float g   = gsum * s.grad_scale;
    const float m1  = __builtin_fmaf(s.beta1, m, s.omb1 * g);
    const float v1  = __builtin_fmaf(s.beta2, v, s.omb2 * (g * g));
    const float den = __builtin_fmaf(__builtin_sqrtf(v1), s.rsqrt_bc2, s.eps);
    const float t0  = __builtin_fmaf(-s.lrwd, theta, theta);
    theta_o         = __builtin_fmaf(-s.step_size, m1 / den, t0);
    m_o             = m1;
    v_o             = v1;
}

// ------------------------------------------------------------------ tile loop

// Every array of this path is streamed once per launch and is far larger than the
// caches, so all vector accesses carry the non-temporal hint (measured: +5 % on the
// committed step at 875M elements).
template <class T>
__device__ __forceinline__ T ld(const T* p)
{
    return __builtin_nontemporal_load(p);
}

template <class T>
__device__ __forceinline__ void st(T* p, T x)
{
    __builtin_nontemporal_store(x, p);
}

// The same store with system scope on top of the non-temporal hint (sc1 nt): the line is
// written through instead of waiting in the L2 for its write-back.  Measured at 875M elements
// against st(): stash 4.13 -> 4.09 ms, second micro-batch + publish 6.11 -> 6.05, committed
// step 3.78 -> 3.73, estimate 2.20 -> 2.19; the two reduce kernels are the exception (reduce +
// commit 5.89 -> 5.95 with it on the state, the output or both), so they keep st().
// s_nop: the store's data registers must not be rewritten in the cycle after it, and the
// compiler does not see inside the asm.
template <class T>
__device__ __forceinline__ void st_through(T* p, T x)
{
    static_assert(sizeof(T) == 16 || sizeof(T) == 8, "vector stores only");
    if constexpr (sizeof(T) == 16)
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(x) : "memory");
    else
        asm volatile("global_store_dwordx2 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(x) : "memory");
}

// Op supplies: kElems (elements per vector: 4, or 8 for all-bf16 kernels); optionally
//              kMaxVectors (most vectors in flight per thread in stream_kernel, default 4;
//              0: the Op is only ever run by flat_kernel); struct In;
//              In load(int64_t vec) const; void apply(int64_t vec, const In&) const;
//              void scalar(int64_t elem) const;
//              struct Shared; static Op make(const BatchPtrs&, int worker, const Shared&)
//              (accumulation Ops only).

// Pointer table of a batched launch: a, b, c are the (up to) three arrays of the Op, one
// entry per worker.
struct BatchPtrs {
    void*       a[kBatchMax];
    const void* b[kBatchMax];
    const void* c[kBatchMax];
};

template <class O>
struct Single {
    typedef O Op;
    O         op;
    __device__ __forceinline__ const O& get(unsigned) const { return op; }
};

template <class O>
struct Batch {
    typedef O          Op;
    BatchPtrs          tab;
    typename O::Shared shared;   // what all workers' Ops have in common (e.g. the output layout)
    __device__ __forceinline__ O get(unsigned worker) const
    {
        return O::make(tab, (int)worker, shared);
    }
};

struct NoShared {};

template <int U, class Src>
__global__ void __launch_bounds__(kMaxThreads) stream_kernel(const Src src, const int64_t nvec,
                                                             const int64_t ntiles, const int64_t n)
{
    typedef typename Src::Op Op;
    const Op                 op   = src.get(blockIdx.y);
    const int64_t            tile = (int64_t)blockDim.x * U;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t   base = t * tile + threadIdx.x;
        typename Op::In in[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * blockDim.x;
            if (i < nvec) in[u] = op.load(i);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * blockDim.x;
            if (i < nvec) op.apply(i, in[u]);
        }
    }
    if (blockIdx.x == 0) {
        const int64_t j = nvec * Op::kElems + threadIdx.x;
        if (j < n) op.scalar(j);
    }
}

// One vector per thread, one tile per workgroup, no loop: the shape that measured
// fastest for these streams (the hardware's workgroup dispatcher does the striding).
template <class Src>
__global__ void __launch_bounds__(kMaxThreads) flat_kernel(const Src src, const int64_t nvec,
                                                           const int64_t n)
{
    typedef typename Src::Op Op;
    const Op                 op = src.get(blockIdx.y);
    const int64_t            i  = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nvec) op.apply(i, op.load(i));
    if (blockIdx.x == 0) {
        const int64_t j = nvec * Op::kElems + threadIdx.x;
        if (j < n) op.scalar(j);
    }
}

// ------------------------------------------------------------------ accumulate

template <bool INIT>
struct AccumulateOp {
    static constexpr int kElems = 4;
    float*          acc;
    const uint16_t* grad;
    typedef NoShared Shared;
    static __device__ __forceinline__ AccumulateOp make(const BatchPtrs& t, int w, const Shared&)
    {
        return AccumulateOp{static_cast<float*>(t.a[w]), static_cast<const uint16_t*>(t.b[w])};
    }
    struct In {
        f4 a;
        u2 g;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.g = ld(reinterpret_cast<const u2*>(grad) + i);
        if (!INIT) in.a = ld(reinterpret_cast<const f4*>(acc) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        const f4 g = unpack_bf16x4(in.g);
        st_through(reinterpret_cast<f4*>(acc) + i, INIT ? g : in.a + g);
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        const float g = __uint_as_float((uint32_t)grad[j] << 16);
        acc[j]        = INIT ? g : acc[j] + g;
    }
};

// Last micro-batch of an accumulation fused with the publish: comm = bf16(acc + grad)
// (INIT: comm = bf16(grad)).  KEEP also stores the fp32 sum back to acc.  OB: comm has a
// blocked layout (the workers' communication buffers interleaved block by block in one buffer).
template <bool INIT, bool KEEP, bool OB = false>
struct AccumulatePublishOp {
    static constexpr int kElems = 4;
    float*          acc;
    const uint16_t* grad;
    uint16_t*       comm;
    StateAddr<OB>   oat;
    typedef StateAddr<OB> Shared;
    // batched form: the accumulator is only read (KEEP is not offered there)
    static __device__ __forceinline__ AccumulatePublishOp make(const BatchPtrs& t, int w,
                                                               const Shared& sh)
    {
        return AccumulatePublishOp{const_cast<float*>(static_cast<const float*>(t.c[w])),
                                   static_cast<const uint16_t*>(t.b[w]),
                                   static_cast<uint16_t*>(t.a[w]), sh};
    }
    struct In {
        f4 a;
        u2 g;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.g = ld(reinterpret_cast<const u2*>(grad) + i);
        if (!INIT) in.a = ld(reinterpret_cast<const f4*>(acc) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        const f4 g = unpack_bf16x4(in.g);
        const f4 s = INIT ? g : in.a + g;
        if (KEEP) st_through(reinterpret_cast<f4*>(acc) + i, s);
        st_through(reinterpret_cast<u2*>(comm) + oat.vec(i), pack_bf16x4(s));
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        const float g = __uint_as_float((uint32_t)grad[j] << 16);
        const float s = INIT ? g : acc[j] + g;
        if (KEEP) acc[j] = s;
        comm[oat.elem(j)] = (uint16_t)to_bf16_bits(s);
    }
};

// ------------------------------------------------------------------ first / second micro-batch

// After the first micro-batch of an accumulation the accumulator equals that gradient, which
// is exactly representable in bf16: it is kept as a bf16 "stash" (2 bytes written instead of
// 4, 2 read back instead of 4).  All-bf16 kernels move 8 elements (16 bytes) per lane.

// a NaN in either half-word gets its quiet bit, as the fp32 -> bf16 rounding would give it
__device__ __forceinline__ uint32_t quiet_bf16x2(uint32_t p)
{
    const uint32_t lo = ((p & 0x00007FFFu) > 0x00007F80u) ? 0x00000040u : 0u;
    const uint32_t hi = ((p & 0x7FFF0000u) > 0x7F800000u) ? 0x00400000u : 0u;
    return p | lo | hi;
}

// stash = grad, or (QUIET) comm = bf16(float(grad)) for a one-micro-batch accumulation.
// An 8-element vector is two consecutive 4-element vectors of the (possibly blocked) output.
template <bool QUIET, bool OB = false>
struct StashOp {
    static constexpr int kElems = 8;
    uint16_t*            dst;
    const uint16_t*      src;
    StateAddr<OB>        oat;
    typedef StateAddr<OB> Shared;
    static __device__ __forceinline__ StashOp make(const BatchPtrs& t, int w, const Shared& sh)
    {
        return StashOp{static_cast<uint16_t*>(t.a[w]), static_cast<const uint16_t*>(t.b[w]), sh};
    }
    struct In {
        u4 x;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.x = ld(reinterpret_cast<const u4*>(src) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        u4 x = in.x;
        if (QUIET) x = (u4){quiet_bf16x2(x.x), quiet_bf16x2(x.y), quiet_bf16x2(x.z), quiet_bf16x2(x.w)};
        st_through(reinterpret_cast<u4*>(reinterpret_cast<u2*>(dst) + oat.vec(2 * i)), x);
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        const uint32_t h = src[j];
        dst[oat.elem(j)] = (uint16_t)(QUIET ? (quiet_bf16x2(h) & 0xFFFFu) : h);
    }
};

// second micro-batch: acc = float(stash) + float(grad), fp32 accumulator from here on
struct SecondOp {
    static constexpr int kElems = 4;
    float*               acc;
    const uint16_t*      stash;
    const uint16_t*      grad;
    typedef NoShared Shared;
    static __device__ __forceinline__ SecondOp make(const BatchPtrs& t, int w, const Shared&)
    {
        return SecondOp{static_cast<float*>(t.a[w]), static_cast<const uint16_t*>(t.c[w]),
                        static_cast<const uint16_t*>(t.b[w])};
    }
    struct In {
        u2 s, g;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.s = ld(reinterpret_cast<const u2*>(stash) + i);
        in.g = ld(reinterpret_cast<const u2*>(grad) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        st_through(reinterpret_cast<f4*>(acc) + i, unpack_bf16x4(in.s) + unpack_bf16x4(in.g));
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        acc[j] = __uint_as_float((uint32_t)stash[j] << 16) + __uint_as_float((uint32_t)grad[j] << 16);
    }
};

// second and last micro-batch fused with the publish: comm = bf16(float(stash) + float(grad))
template <bool OB = false>
struct SecondPublishOp {
    static constexpr int kElems = 8;
    uint16_t*            comm;
    const uint16_t*      stash;
    const uint16_t*      grad;
    StateAddr<OB>        oat;
    typedef StateAddr<OB> Shared;
    static __device__ __forceinline__ SecondPublishOp make(const BatchPtrs& t, int w,
                                                           const Shared& sh)
    {
        return SecondPublishOp{static_cast<uint16_t*>(t.a[w]), static_cast<const uint16_t*>(t.c[w]),
                               static_cast<const uint16_t*>(t.b[w]), sh};
    }
    struct In {
        u4 s, g;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.s = ld(reinterpret_cast<const u4*>(stash) + i);
        in.g = ld(reinterpret_cast<const u4*>(grad) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        const u2 lo = pack_bf16x4(unpack_bf16x4((u2){in.s.x, in.s.y}) + unpack_bf16x4((u2){in.g.x, in.g.y}));
        const u2 hi = pack_bf16x4(unpack_bf16x4((u2){in.s.z, in.s.w}) + unpack_bf16x4((u2){in.g.z, in.g.w}));
        st_through(reinterpret_cast<u4*>(reinterpret_cast<u2*>(comm) + oat.vec(2 * i)),
           (u4){lo.x, lo.y, hi.x, hi.y});
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        comm[oat.elem(j)] = (uint16_t)to_bf16_bits(__uint_as_float((uint32_t)stash[j] << 16) +
                                                   __uint_as_float((uint32_t)grad[j] << 16));
    }
};

// ------------------------------------------------------------------ cast

template <bool OB = false>
struct CastOp {
    static constexpr int kElems = 4;
    uint16_t*     out;
    const float*  src;
    StateAddr<OB> oat;
    typedef StateAddr<OB> Shared;
    static __device__ __forceinline__ CastOp make(const BatchPtrs& t, int w, const Shared& sh)
    {
        return CastOp{static_cast<uint16_t*>(t.a[w]), static_cast<const float*>(t.c[w]), sh};
    }
    struct In {
        f4 x;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.x = ld(reinterpret_cast<const f4*>(src) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        st_through(reinterpret_cast<u2*>(out) + oat.vec(i), pack_bf16x4(in.x));
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        out[oat.elem(j)] = (uint16_t)to_bf16_bits(src[j]);
    }
};

// ------------------------------------------------------------------ reduce

template <int WMAX>
struct ShardPtrs {
    const void* p[WMAX];
};

// Sum of up to WMAX worker shards per launch, ascending worker order.  ACC: start
// from the value already in gsum, else from shard 0 as it is.  SB: the shards have a blocked
// layout of their own (the workers' buffers interleaved block by block in one buffer).
template <int WMAX, bool BF16, bool ACC, bool BLOCKED, bool SB = false>
struct ReduceOp {
    static constexpr int kElems = 4;
    // vectors in flight per thread in the looping kernel: fp32 shards hold too many loads for
    // more than 2 (they would spill); the wide form exists as the flat kernel only (0)
    static constexpr int kMaxVectors = WMAX > kReduceChunk ? 0 : BF16 ? 4 : 2;
    float*             gsum;
    ShardPtrs<WMAX>    shards;
    int                workers;  // 1 .. WMAX
    StateAddr<BLOCKED> at;       // layout of gsum
    StateAddr<SB>      sat;      // layout of every shard
    struct In {
        f4 s;
        f4 x[BF16 ? 1 : WMAX];
        u2 b[BF16 ? WMAX : 1];
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        if (ACC) in.s = ld(reinterpret_cast<const f4*>(gsum) + at.vec(i));
#pragma unroll
        for (int w = 0; w < WMAX; ++w) {
            if (w < workers) {
                if (BF16)
                    in.b[w] = ld(reinterpret_cast<const u2*>(shards.p[w]) + sat.vec(i));
                else
                    in.x[w] = ld(reinterpret_cast<const f4*>(shards.p[w]) + sat.vec(i));
            }
        }
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        f4 s = in.s;
#pragma unroll
        for (int w = 0; w < WMAX; ++w) {
            if (w < workers) {
                const f4 x = BF16 ? unpack_bf16x4(in.b[w]) : in.x[w];
                s          = (!ACC && w == 0) ? x : s + x;
            }
        }
        st(reinterpret_cast<f4*>(gsum) + at.vec(i), s);
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        const int64_t a = at.elem(j), b = sat.elem(j);
        float         s = ACC ? gsum[a] : 0.0f;
        // unrolled, so that the pointer table is indexed by constants (it lives in the kernel
        // arguments; a run-time index would copy it to private memory)
#pragma unroll
        for (int w = 0; w < WMAX; ++w) {
            if (w < workers) {
                const float x =
                    BF16 ? __uint_as_float((uint32_t)static_cast<const uint16_t*>(shards.p[w])[b] << 16)
                         : static_cast<const float*>(shards.p[w])[b];
                s = (!ACC && w == 0) ? x : s + x;
            }
        }
        gsum[a] = s;
    }
};

// ------------------------------------------------------------------ estimate / commit

__device__ __forceinline__ void adamw_vec(f4 t, f4 m, f4 v, f4 g, const AdamScalars& s, f4& to,
                                          f4& mo, f4& vo)
{
    float a[4], b[4], c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) adamw_elem(t[k], m[k], v[k], g[k], s, a[k], b[k], c[k]);
    to = (f4){a[0], a[1], a[2], a[3]};
    mo = (f4){b[0], b[1], b[2], b[3]};
    vo = (f4){c[0], c[1], c[2], c[3]};
}

// COMMIT: write theta, m, v in place.  OUT_F32 / OUT_BF16: extra (planar) outputs of the
// new theta.  BLOCKED: theta, m, v, gsum share a blocked layout.
template <bool COMMIT, bool OUT_F32, bool OUT_BF16, bool BLOCKED, class SC = ScalarsByValue>
struct AdamOp {
    static constexpr int kElems = 4;
    const float*       theta;
    const float*       m;
    const float*       v;
    const float*       gsum;
    float*             theta_w;  // COMMIT: == theta
    float*             m_w;
    float*             v_w;
    float*             out_f32;
    uint16_t*          out_bf16;
    SC                 s;
    StateAddr<BLOCKED> at;
    struct In {
        f4 t, m, v, g;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        const int64_t a = at.vec(i);
        In            in;
        in.t = ld(reinterpret_cast<const f4*>(theta) + a);
        in.m = ld(reinterpret_cast<const f4*>(m) + a);
        in.v = ld(reinterpret_cast<const f4*>(v) + a);
        in.g = ld(reinterpret_cast<const f4*>(gsum) + a);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        f4 t, mm, vv;
        adamw_vec(in.t, in.m, in.v, in.g, s.get(), t, mm, vv);
        if (COMMIT) {
            const int64_t a = at.vec(i);
            st_through(reinterpret_cast<f4*>(theta_w) + a, t);
            st_through(reinterpret_cast<f4*>(m_w) + a, mm);
            st_through(reinterpret_cast<f4*>(v_w) + a, vv);
        }
        if (OUT_F32) st_through(reinterpret_cast<f4*>(out_f32) + i, t);
        if (OUT_BF16) st_through(reinterpret_cast<u2*>(out_bf16) + i, pack_bf16x4(t));
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        const int64_t a = at.elem(j);
        float         t, mm, vv;
        adamw_elem(theta[a], m[a], v[a], gsum[a], s.get(), t, mm, vv);
        if (COMMIT) {
            theta_w[a] = t;
            m_w[a]     = mm;
            v_w[a]     = vv;
        }
        if (OUT_F32) out_f32[j] = t;
        if (OUT_BF16) out_bf16[j] = (uint16_t)to_bf16_bits(t);
    }
};

// ------------------------------------------------------------------ reduce fused with the step

// The owner-side reduction of up to WMAX worker shards folded into the AdamW step:
// the gradient sum is formed in registers (same order as ReduceOp), optionally stored to
// gsum (stage 1 keeps it for stage 2), and consumed by the update in the same pass.
template <bool COMMIT, bool BF16, bool ACC, bool WRITE_GSUM, bool OUT_F32, bool OUT_BF16,
          bool BLOCKED, bool SB = false, class SC = ScalarsByValue, int WMAX = kReduceChunk>
struct ReduceAdamOp {
    static constexpr int kElems = 4;
    static constexpr int kMaxVectors = WMAX > kReduceChunk ? 0 : BF16 ? 4 : 2;
    const float*       theta;
    const float*       m;
    const float*       v;
    float*             gsum;  // read when ACC, written when WRITE_GSUM
    ShardPtrs<WMAX>    shards;
    int                workers;
    float*             theta_w;
    float*             m_w;
    float*             v_w;
    float*             out_f32;
    uint16_t*          out_bf16;
    SC                 s;
    StateAddr<BLOCKED> at;
    StateAddr<SB>      sat;   // layout of every shard
    struct In {
        f4 t, m, v, g;
        f4 x[BF16 ? 1 : WMAX];
        u2 b[BF16 ? WMAX : 1];
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        const int64_t a = at.vec(i);
        In            in;
        in.t = ld(reinterpret_cast<const f4*>(theta) + a);
        in.m = ld(reinterpret_cast<const f4*>(m) + a);
        in.v = ld(reinterpret_cast<const f4*>(v) + a);
        if (ACC) in.g = ld(reinterpret_cast<const f4*>(gsum) + a);
#pragma unroll
        for (int w = 0; w < WMAX; ++w) {
            if (w < workers) {
                if (BF16)
                    in.b[w] = ld(reinterpret_cast<const u2*>(shards.p[w]) + sat.vec(i));
                else
                    in.x[w] = ld(reinterpret_cast<const f4*>(shards.p[w]) + sat.vec(i));
            }
        }
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        const int64_t a = at.vec(i);
        f4            g = in.g;
#pragma unroll
        for (int w = 0; w < WMAX; ++w) {
            if (w < workers) {
                const f4 x = BF16 ? unpack_bf16x4(in.b[w]) : in.x[w];
                g          = (!ACC && w == 0) ? x : g + x;
            }
        }
        if (WRITE_GSUM) st(reinterpret_cast<f4*>(gsum) + a, g);
        f4 t, mm, vv;
        adamw_vec(in.t, in.m, in.v, g, s.get(), t, mm, vv);
        if (COMMIT) {
            st(reinterpret_cast<f4*>(theta_w) + a, t);
            st(reinterpret_cast<f4*>(m_w) + a, mm);
            st(reinterpret_cast<f4*>(v_w) + a, vv);
        }
        if (OUT_F32) st(reinterpret_cast<f4*>(out_f32) + i, t);
        if (OUT_BF16) st(reinterpret_cast<u2*>(out_bf16) + i, pack_bf16x4(t));
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        const int64_t a = at.elem(j), b = sat.elem(j);
        float         g = ACC ? gsum[a] : 0.0f;
#pragma unroll
        for (int w = 0; w < WMAX; ++w) {
            if (w < workers) {
                const float x =
                    BF16 ? __uint_as_float((uint32_t)static_cast<const uint16_t*>(shards.p[w])[b] << 16)
                         : static_cast<const float*>(shards.p[w])[b];
                g = (!ACC && w == 0) ? x : g + x;
            }
        }
        if (WRITE_GSUM) gsum[a] = g;
        float t, mm, vv;
        adamw_elem(theta[a], m[a], v[a], g, s.get(), t, mm, vv);
        if (COMMIT) {
            theta_w[a] = t;
            m_w[a]     = mm;
            v_w[a]     = vv;
        }
        if (OUT_F32) out_f32[j] = t;
        if (OUT_BF16) out_bf16[j] = (uint16_t)to_bf16_bits(t);
    }
};

// ------------------------------------------------------------------ SGD as Opt

// Plain (stochastic) gradient descent with decoupled decay, the Opt of the paper's
// convergence propositions: theta' = theta - lr wd theta - lr g,  g = gsum / count.
struct SgdScalars {
    float grad_scale;
    float lr;
    float lrwd;
};

__device__ __forceinline__ float sgd_elem(float theta, float gsum, const SgdScalars& s)
{
    const float g  = gsum * s.grad_scale;
    const float t0 = __builtin_fmaf(-s.lrwd, theta, theta);
    return __builtin_fmaf(-s.lr, g, t0);
}

template <bool COMMIT, bool OUT_F32, bool OUT_BF16>
struct SgdOp {
    static constexpr int kElems = 4;
    const float* theta;
    const float* gsum;
    float*       theta_w;
    float*       out_f32;
    uint16_t*    out_bf16;
    SgdScalars   s;
    struct In {
        f4 t, g;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.t = ld(reinterpret_cast<const f4*>(theta) + i);
        in.g = ld(reinterpret_cast<const f4*>(gsum) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        const f4 t = {sgd_elem(in.t.x, in.g.x, s), sgd_elem(in.t.y, in.g.y, s),
                      sgd_elem(in.t.z, in.g.z, s), sgd_elem(in.t.w, in.g.w, s)};
        if (COMMIT) st_through(reinterpret_cast<f4*>(theta_w) + i, t);
        if (OUT_F32) st_through(reinterpret_cast<f4*>(out_f32) + i, t);
        if (OUT_BF16) st_through(reinterpret_cast<u2*>(out_bf16) + i, pack_bf16x4(t));
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        const float t = sgd_elem(theta[j], gsum[j], s);
        if (COMMIT) theta_w[j] = t;
        if (OUT_F32) out_f32[j] = t;
        if (OUT_BF16) out_bf16[j] = (uint16_t)to_bf16_bits(t);
    }
};

// ------------------------------------------------------------------ bandwidth probes

// Not part of the method: the access patterns of the step kernels without their arithmetic,
// to measure on the same device what the memory system gives (reported beside the kernels).
struct ProbeCopyOp {
    static constexpr int kElems = 4;
    float*               dst;
    const float*         src;
    struct In {
        f4 x;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.x = ld(reinterpret_cast<const f4*>(src) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        st_through(reinterpret_cast<f4*>(dst) + i, in.x);
    }
    __device__ __forceinline__ void scalar(int64_t j) const { dst[j] = src[j]; }
};

// two streams read, one written (out = a ^ b, 16 bytes per lane): the access pattern of a
// second micro-batch, with no floating point; what acco_hbm_classify times
struct ProbePairOp {
    static constexpr int kElems = 4;   // "elements" here are 4-byte words: one u4 per lane
    uint32_t*            out;
    const uint32_t*      a;
    const uint32_t*      b;
    struct In {
        u4 a, b;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.a = ld(reinterpret_cast<const u4*>(a) + i);
        in.b = ld(reinterpret_cast<const u4*>(b) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        st_through(reinterpret_cast<u4*>(out) + i, in.a ^ in.b);
    }
    __device__ __forceinline__ void scalar(int64_t j) const { out[j] = a[j] ^ b[j]; }
};

// four fp32 arrays read, three of them written back in place (a += d, b += d, c += d)
struct ProbeTriadOp {
    static constexpr int kElems = 4;
    float*               a;
    float*               b;
    float*               c;
    const float*         d;
    struct In {
        f4 a, b, c, d;
    };
    __device__ __forceinline__ In load(int64_t i) const
    {
        In in;
        in.a = ld(reinterpret_cast<const f4*>(a) + i);
        in.b = ld(reinterpret_cast<const f4*>(b) + i);
        in.c = ld(reinterpret_cast<const f4*>(c) + i);
        in.d = ld(reinterpret_cast<const f4*>(d) + i);
        return in;
    }
    __device__ __forceinline__ void apply(int64_t i, const In& in) const
    {
        st_through(reinterpret_cast<f4*>(a) + i, in.a + in.d);
        st_through(reinterpret_cast<f4*>(b) + i, in.b + in.d);
        st_through(reinterpret_cast<f4*>(c) + i, in.c + in.d);
    }
    __device__ __forceinline__ void scalar(int64_t j) const
    {
        a[j] += d[j];
        b[j] += d[j];
        c[j] += d[j];
    }
};

}  // namespace acco
