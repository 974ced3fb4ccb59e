/*
 * Host fill routines of the synthetic input generator (see synth_core.h).
 * Built by gcc into libsynth_host.so; loaded through ctypes.
 * out[i] holds stream element j0 + i, so a slice equals the same slice of the
 * full buffer.
 */
#include "synth_core.h"

#define SYNTH_EXPORT __attribute__((visibility("default")))

SYNTH_EXPORT uint64_t synth_host_stream_key(uint64_t seed, uint32_t kind, uint32_t round,
                                            uint32_t stage, uint32_t worker, uint32_t mb)
{
    return synth_stream_key(seed, kind, round, stage, worker, mb);
}

SYNTH_EXPORT uint64_t synth_host_hash(uint64_t key, int64_t j) { return synth_hash(key, j); }

SYNTH_EXPORT double synth_host_ih4_sigma(void) { return SYNTH_IH4_SIGMA; }

SYNTH_EXPORT void synth_host_fill_normal_f32(float* out, int64_t j0, int64_t n, uint64_t key,
                                             float scale)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = synth_normal_f32(key, j0 + i, scale);
}

SYNTH_EXPORT void synth_host_fill_uniform_f32(float* out, int64_t j0, int64_t n, uint64_t key,
                                              float scale)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = synth_uniform_f32(key, j0 + i, scale);
}

SYNTH_EXPORT void synth_host_fill_grad_bf16(uint16_t* out, int64_t j0, int64_t n,
                                            const synth_grad_spec* sp)
{
    synth_grad_spec s = *sp;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = synth_grad_bf16(&s, j0 + i);
}
