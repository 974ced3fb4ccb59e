/*
 * CPU ORACLE for the ACCO per-shard optimizer path.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP library and to be timed beside it.  Nothing in the
 * product path may call it, and it shares no code with the HIP library.
 *
 * Plain scalar C, one element at a time, in the order the definitions are
 * written.  Build: gcc -O2 -ffp-contract=off -fno-fast-math (no FTZ/DAZ), so
 * every fp32 operation below is a single IEEE-754 binary32 operation.
 *
 * What is computed, and where the paper defines it:
 *   accumulate      g_i <- g_i + grad(micro-batch)            Alg. 1, computation stream
 *   publish / cast  fp32 -> bf16 (comm buffer, parameters)    Sec. 4.2 (bf16 params, grads,
 *                                                              comm buffers; fp32 sharded states)
 *   reduce          owner's slice of sum_i g_i                Alg. 1, Reduce_Scatter lines
 *   estimate        theta~(t+1) = Opt(theta(t), sum g~/sum N~)   eq. (ACCO) stage (1)
 *   commit          theta(t+1) = Opt(theta(t), (sum g + sum g~)/(sum N + sum N~))
 *                                                              eq. (ACCO) stage (2)
 *   Opt = AdamW with bias correction (Sec. 4.2; hyper-parameters App. C tables).
 *
 * Two forms of the AdamW element update are provided:
 *   *_f64  the textbook definition written out in binary64 on the fp32-stored
 *          state, results rounded once to fp32 (the reference value);
 *   *_f32  the same update in binary32, each operation individually rounded,
 *          with the bias corrections folded into host scalars (the precision
 *          the paper fixes for the sharded states).
 * Readings taken where the paper is silent: the estimate does not advance m, v or
 * the step index; epsilon is added after the bias-corrected square root; the decay
 * multiplies theta(t); the gradient sum is divided by the total micro-batch count.
 * Each is repeated at the function it concerns.
 *
 * Pins: every function here is pinned by tests that do not call back into this
 * file's formulas (closed forms, exhaustive bf16 tables, torch CPU routines,
 * exact rational arithmetic, brute force).  No function is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_EXPORT __attribute__((visibility("default")))

typedef struct oracle_hyper {
    double lr, beta1, beta2, eps, weight_decay;
} oracle_hyper;

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1 };

static int g_threads = 1;

/* number of OpenMP threads the array loops use (elements are independent, so
 * threading changes no result) */
ORACLE_EXPORT void oracle_set_threads(int t)
{
    g_threads = t < 1 ? 1 : t;
}

ORACLE_EXPORT int oracle_get_threads(void)
{
    return g_threads;
}

ORACLE_EXPORT int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ bf16 <-> fp32 */

/* bf16 is the upper half of a binary32 word: widening is exact. */
ORACLE_EXPORT float oracle_bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float    f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round to nearest, ties to even, on the upper 16 bits.  NaN stays NaN (quiet
 * bit set, sign kept); infinities are kept; finite values beyond the largest
 * bf16 round to infinity. */
ORACLE_EXPORT uint16_t oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* ------------------------------------------------------------------ accumulate */

/* Alg. 1, computation stream: g_i <- g_i + grad.  `init` starts a new
 * accumulation (the buffer is overwritten, which is "zeroed then added" except
 * that it keeps the sign of a -0 gradient). */
ORACLE_EXPORT void oracle_accumulate(float* acc, const uint16_t* grad_bf16, int64_t n, int init)
{
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) {
        float g = oracle_bf16_to_f32(grad_bf16[j]);
        acc[j]  = init ? g : acc[j] + g;
    }
}

/* The same accumulation with the running sum itself held in bf16, which is the
 * precision the paper's experimental setup (Sec. 4, "gradient accumulation and
 * communication buffers" in bf16) gives the buffer: the two bf16 values are added
 * exactly-rounded in binary32 and the sum is rounded to bf16, nearest-even.
 * (A binary32 sum of two bf16 values followed by the bf16 rounding equals the
 * directly rounded bf16 sum: 24 bits are more than 2*8+2.) */
ORACLE_EXPORT void oracle_accumulate_bf16(uint16_t* acc_bf16, const uint16_t* grad_bf16, int64_t n,
                                          int init)
{
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) {
        if (init) { acc_bf16[j] = grad_bf16[j]; continue; }
        float s = oracle_bf16_to_f32(acc_bf16[j]) + oracle_bf16_to_f32(grad_bf16[j]);
        acc_bf16[j] = oracle_f32_to_bf16(s);
    }
}

/* Buffer_i <- g_i (bf16 communication buffer) and the bf16 parameter copy that
 * the All_Gather distributes. */
ORACLE_EXPORT void oracle_cast(uint16_t* out_bf16, const float* in, int64_t n)
{
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) out_bf16[j] = oracle_f32_to_bf16(in[j]);
}

/* ------------------------------------------------------------------ reduce */

/* Owner's slice of the Reduce_Scatter: sum over workers in ascending worker
 * order, in fp32.  accumulate != 0 adds onto the sum already in gsum (stage 2
 * adds the second-half gradients to the retained first-half sum). */
ORACLE_EXPORT void oracle_reduce(float* gsum, const void* const* shards, int workers, int dtype,
                                 int64_t n, int accumulate)
{
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) {
        float s = accumulate ? gsum[j] : 0.0f;
        for (int w = 0; w < workers; ++w) {
            float x = dtype == ORACLE_BF16 ? oracle_bf16_to_f32(((const uint16_t*)shards[w])[j])
                                           : ((const float*)shards[w])[j];
            /* the first term of a fresh sum is taken as is (0 + x would turn -0 into +0) */
            s = (!accumulate && w == 0) ? x : s + x;
        }
        gsum[j] = s;
    }
}

/* ------------------------------------------------------------------ AdamW, one element */

/* Textbook AdamW with bias correction, binary64 arithmetic, at update index
 * `step` (1-based), on the gradient sum divided by the total count. */
static void adamw_elem_f64(float theta, float m, float v, float gsum, double count,
                           const oracle_hyper* hp, double bc1, double bc2, float* theta_o,
                           float* m_o, float* v_o)
{
    /* bc1 = 1 - beta1^step, bc2 = 1 - beta2^step: the same for every element of a step */
    double g     = (double)gsum / count;
    double m1    = hp->beta1 * (double)m + (1.0 - hp->beta1) * g;
    double v1    = hp->beta2 * (double)v + (1.0 - hp->beta2) * g * g;
    double m_hat = m1 / bc1;
    double v_hat = v1 / bc2;
    double th    = (double)theta;
    double t1    = th - hp->lr * hp->weight_decay * th - hp->lr * m_hat / (sqrt(v_hat) + hp->eps);
    *theta_o     = (float)t1;
    *m_o         = (float)m1;
    *v_o         = (float)v1;
}

/* Host scalars of the binary32 form: computed in binary64, rounded once. */
typedef struct folded {
    float grad_scale; /* 1 / count                       */
    float beta1, beta2, omb1, omb2;
    float step_size;  /* lr / (1 - beta1^step)           */
    float rsqrt_bc2;  /* 1 / sqrt(1 - beta2^step)        */
    float lrwd;       /* lr * weight_decay               */
    float eps;
} folded;

static folded fold(const oracle_hyper* hp, int64_t step, int64_t count)
{
    folded f;
    double bc1   = 1.0 - pow(hp->beta1, (double)step);
    double bc2   = 1.0 - pow(hp->beta2, (double)step);
    f.grad_scale = (float)(1.0 / (double)count);
    f.beta1      = (float)hp->beta1;
    f.beta2      = (float)hp->beta2;
    f.omb1       = (float)(1.0 - hp->beta1);
    f.omb2       = (float)(1.0 - hp->beta2);
    f.step_size  = (float)(hp->lr / bc1);
    f.rsqrt_bc2  = (float)(1.0 / sqrt(bc2));
    f.lrwd       = (float)(hp->lr * hp->weight_decay);
    f.eps        = (float)hp->eps;
    return f;
}

/* The same update in binary32, one rounding per line-level operation, in this
 * order; fmaf is the single-rounding fused multiply-add.  The decay is applied as
 * theta - (lr wd) theta in one fused operation: multiplying by a pre-rounded
 * (1 - lr wd) would bias theta by up to 2^-25 relative on every step. */
static void adamw_elem_f32(float theta, float m, float v, float gsum, const folded* f,
                           float* theta_o, float* m_o, float* v_o)
{
    float g   = gsum * f->grad_scale;
    float m1  = fmaf(f->beta1, m, f->omb1 * g);
    float v1  = fmaf(f->beta2, v, f->omb2 * (g * g));
    float den = fmaf(sqrtf(v1), f->rsqrt_bc2, f->eps);
    float t0  = fmaf(-f->lrwd, theta, theta);
    float t1  = fmaf(-f->step_size, m1 / den, t0);
    *theta_o  = t1;
    *m_o      = m1;
    *v_o      = v1;
}

/* ------------------------------------------------------------------ estimate / commit */

/* eq. (ACCO) stage (1): theta~ = Opt(theta, gsum / count) at update index
 * `step`; theta, m, v are only read.  Either output may be NULL. */
ORACLE_EXPORT void oracle_estimate_f64(const float* theta, const float* m, const float* v,
                                       const float* gsum, float* out_f32, uint16_t* out_bf16,
                                       int64_t n, const oracle_hyper* hp, int64_t step,
                                       int64_t count)
{
    const double bc1 = 1.0 - pow(hp->beta1, (double)step);
    const double bc2 = 1.0 - pow(hp->beta2, (double)step);
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) {
        float t1, m1, v1;
        adamw_elem_f64(theta[j], m[j], v[j], gsum[j], (double)count, hp, bc1, bc2, &t1, &m1,
                       &v1);
        if (out_f32) out_f32[j] = t1;
        if (out_bf16) out_bf16[j] = oracle_f32_to_bf16(t1);
    }
}

ORACLE_EXPORT void oracle_estimate_f32(const float* theta, const float* m, const float* v,
                                       const float* gsum, float* out_f32, uint16_t* out_bf16,
                                       int64_t n, const oracle_hyper* hp, int64_t step,
                                       int64_t count)
{
    const folded f = fold(hp, step, count);
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) {
        float t1, m1, v1;
        adamw_elem_f32(theta[j], m[j], v[j], gsum[j], &f, &t1, &m1, &v1);
        if (out_f32) out_f32[j] = t1;
        if (out_bf16) out_bf16[j] = oracle_f32_to_bf16(t1);
    }
}

/* eq. (ACCO) stage (2): (theta, m, v) <- Opt(theta, m, v, gsum / count) at update
 * index `step`, in place; optional bf16 copy of the new theta.  The caller
 * advances its step counter afterwards. */
ORACLE_EXPORT void oracle_commit_f64(float* theta, float* m, float* v, const float* gsum,
                                     uint16_t* out_bf16, int64_t n, const oracle_hyper* hp,
                                     int64_t step, int64_t count)
{
    const double bc1 = 1.0 - pow(hp->beta1, (double)step);
    const double bc2 = 1.0 - pow(hp->beta2, (double)step);
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) {
        float t1, m1, v1;
        adamw_elem_f64(theta[j], m[j], v[j], gsum[j], (double)count, hp, bc1, bc2, &t1, &m1,
                       &v1);
        theta[j] = t1;
        m[j]     = m1;
        v[j]     = v1;
        if (out_bf16) out_bf16[j] = oracle_f32_to_bf16(t1);
    }
}

ORACLE_EXPORT void oracle_commit_f32(float* theta, float* m, float* v, const float* gsum,
                                     uint16_t* out_bf16, int64_t n, const oracle_hyper* hp,
                                     int64_t step, int64_t count)
{
    const folded f = fold(hp, step, count);
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) {
        float t1, m1, v1;
        adamw_elem_f32(theta[j], m[j], v[j], gsum[j], &f, &t1, &m1, &v1);
        theta[j] = t1;
        m[j]     = m1;
        v[j]     = v1;
        if (out_bf16) out_bf16[j] = oracle_f32_to_bf16(t1);
    }
}

/* ------------------------------------------------------------------ SGD as Opt */

/* The optimizer of the paper's convergence propositions (Prop. GD / Prop. SGD):
 * theta' = theta - lr wd theta - lr g with g = gsum / count.  Binary64 form: the definition;
 * binary32 form: g = gsum * fp32(1/count); t0 = fma(-(lr wd), theta, theta);
 * theta' = fma(-lr, g, t0). */
static float sgd_elem_f64(float theta, float gsum, double count, double lr, double wd)
{
    double th = (double)theta;
    return (float)(th - lr * wd * th - lr * ((double)gsum / count));
}

static float sgd_elem_f32(float theta, float gsum, float grad_scale, float lr, float lrwd)
{
    float g  = gsum * grad_scale;
    float t0 = fmaf(-lrwd, theta, theta);
    return fmaf(-lr, g, t0);
}

/* theta_out may alias theta (commit) or be a separate buffer (estimate); either output may
 * be NULL. */
ORACLE_EXPORT void oracle_sgd_step(const float* theta, const float* gsum, float* theta_out,
                                   uint16_t* out_bf16, int64_t n, double lr, double weight_decay,
                                   int64_t count, int use_f32)
{
    const float gs = (float)(1.0 / (double)count), lrf = (float)lr,
                lw = (float)(lr * weight_decay);
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < n; ++j) {
        float t1 = use_f32 ? sgd_elem_f32(theta[j], gsum[j], gs, lrf, lw)
                           : sgd_elem_f64(theta[j], gsum[j], (double)count, lr, weight_decay);
        if (theta_out) theta_out[j] = t1;
        if (out_bf16) out_bf16[j] = oracle_f32_to_bf16(t1);
    }
}
