/*
 * Seeded, counter-based synthetic input generator: the element at index j of a
 * stream is a pure function of (stream key, j), so any slice of any buffer can be
 * produced on its own, on the host or on the device, with identical bits.
 *
 * This header is the whole generator.  It is compiled twice, by gcc for the host
 * fill routines and by hipcc for the device fill kernels, and holds NONE of the
 * optimizer path's arithmetic: it only manufactures inputs (parameter shards,
 * micro-batch gradients) that the CPU oracle and the HIP library both consume.
 *
 * Every value is built from integer hashing followed by ONE int->fp32 conversion
 * (exact: |int| < 2^24) and ONE fp32 multiply, so host and device agree bit for
 * bit without depending on contraction or library math.
 */
#ifndef ACCO_SYNTH_CORE_H
#define ACCO_SYNTH_CORE_H

#include <stdint.h>

#if defined(__HIPCC__)
#define SYNTH_HD __host__ __device__ static inline
#else
#define SYNTH_HD static inline
#endif

/* Odd 64-bit constants: fractional bits of the golden ratio, sqrt(2), sqrt(3). */
#define SYNTH_C_PHI   0x9E3779B97F4A7C15ULL
#define SYNTH_C_SQRT2 0x6A09E667F3BCC909ULL
#define SYNTH_C_SQRT3 0xBB67AE8584CAA73BULL

/* Standard deviation of the sum of four independent uniforms on {0..65535}:
 * sqrt(4 * (65536^2 - 1) / 12).  Host code divides the wanted std by this. */
#define SYNTH_IH4_SIGMA 37837.22754635364

typedef struct synth_grad_spec {
    uint64_t key;           /* stream key of this micro-batch gradient            */
    float    scale;         /* std / SYNTH_IH4_SIGMA, rounded once to fp32         */
    float    outlier_scale; /* scale used for hash-selected outlier elements       */
    uint32_t outlier_thr;   /* element is an outlier iff hash32 < thr (0 = none)   */
    uint32_t mask_thr;      /* run of elements is zeroed iff hash32 < thr (0=none) */
    uint32_t mask_run;      /* length of a zero run in elements (>= 1)             */
    uint32_t _pad;
    uint64_t mask_key;      /* key of the zero mask (shared by a round's streams)  */
} synth_grad_spec;

/* multiply-xorshift finaliser */
SYNTH_HD uint64_t synth_mix64(uint64_t x)
{
    x ^= x >> 31;
    x *= SYNTH_C_SQRT2;
    x ^= x >> 29;
    x *= SYNTH_C_SQRT3;
    x ^= x >> 32;
    return x;
}

/* key of a stream: which tensor, which round/stage/worker/micro-batch */
SYNTH_HD uint64_t synth_stream_key(uint64_t seed, uint32_t kind, uint32_t round,
                                   uint32_t stage, uint32_t worker, uint32_t microbatch)
{
    uint64_t id = ((uint64_t)(kind & 0xFFu) << 56) | ((uint64_t)(stage & 0xFFu) << 48) |
                  ((uint64_t)(round & 0xFFFFu) << 32) | ((uint64_t)(worker & 0xFFFFu) << 16) |
                  (uint64_t)(microbatch & 0xFFFFu);
    return synth_mix64(synth_mix64(seed + SYNTH_C_PHI) ^ (id * SYNTH_C_PHI));
}

SYNTH_HD uint64_t synth_hash(uint64_t key, int64_t j)
{
    return synth_mix64(key + (uint64_t)j * SYNTH_C_PHI);
}

/* approximate N(0,1)*sigma: centred sum of the four 16-bit lanes of the hash
 * (Irwin-Hall, support +-131070), one exact conversion, one multiply. */
SYNTH_HD float synth_normal_from_hash(uint64_t h, float scale)
{
    int32_t s = (int32_t)(h & 0xFFFFu) + (int32_t)((h >> 16) & 0xFFFFu) +
                (int32_t)((h >> 32) & 0xFFFFu) + (int32_t)(h >> 48) - 131070;
    return (float)s * scale;
}

SYNTH_HD float synth_normal_f32(uint64_t key, int64_t j, float scale)
{
    return synth_normal_from_hash(synth_hash(key, j), scale);
}

/* symmetric uniform on (-a, a): scale = a / 2^24 rounded once to fp32; the odd
 * integer 2u - (2^24 - 1), |.| < 2^24, converts exactly. */
SYNTH_HD float synth_uniform_f32(uint64_t key, int64_t j, float scale)
{
    uint64_t h = synth_hash(key, j);
    int32_t  s = 2 * (int32_t)(h >> 40) - 16777215;
    return (float)s * scale;
}

/* fp32 -> bf16 bits, round to nearest even (generator inputs are always finite) */
SYNTH_HD uint16_t synth_to_bf16(float x)
{
    union { float f; uint32_t u; } c;
    c.f = x;
    uint32_t r = c.u + 0x7FFFu + ((c.u >> 16) & 1u);
    return (uint16_t)(r >> 16);
}

/* one element of a bf16 micro-batch gradient */
SYNTH_HD uint16_t synth_grad_bf16(const synth_grad_spec* sp, int64_t j)
{
    if (sp->mask_thr != 0u) {
        uint64_t run = (uint64_t)j / (uint64_t)sp->mask_run;
        uint32_t hm  = (uint32_t)(synth_hash(sp->mask_key, (int64_t)run) >> 32);
        if (hm < sp->mask_thr) return (uint16_t)0;
    }
    uint64_t h     = synth_hash(sp->key, j);
    float    scale = sp->scale;
    if (sp->outlier_thr != 0u) {
        uint32_t ho = (uint32_t)(synth_mix64(h ^ SYNTH_C_PHI) >> 32);
        if (ho < sp->outlier_thr) scale = sp->outlier_scale;
    }
    return synth_to_bf16(synth_normal_from_hash(h, scale));
}

#endif /* ACCO_SYNTH_CORE_H */
