/* One ACCO round of a shard owner driven from plain C: memory from hipMalloc, a stream from
 * hipStreamCreate, the library's entry points and nothing else (no Python, no torch in the
 * process).  The round is run twice on copies of the same state - once through the five base
 * entry points (Alg. 1, communication stream, one call per line), once through the fused forms -
 * and both results go to the output file, where the test compares them with the oracle.
 *
 * usage: round_from_c IN OUT
 * IN : int64 n, W, K, step0; double lr, beta1, beta2, eps, wd; float theta[n], m[n], v[n];
 *      uint16 grads[2][W][K][n] (bf16 bit patterns; stage, worker, micro-batch)
 * OUT: for each of the two paths: uint16 theta_tilde_bf16[n]; float theta[n], m[n], v[n];
 *      uint16 theta_bf16[n]; int64 step, total
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "acco.h"

#define MAXW 16
#define MAXK 8

#define HIP(call)                                                                       \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess) {                                                         \
            fprintf(stderr, "line %d: %s: %s\n", __LINE__, #call, hipGetErrorString(e_)); \
            return 2;                                                                   \
        }                                                                               \
    } while (0)

#define ACCO(call)                                                                      \
    do {                                                                                \
        int s_ = (call);                                                                \
        if (s_ != ACCO_OK) {                                                            \
            fprintf(stderr, "line %d: %s: %s\n", __LINE__, #call, acco_status_string(s_)); \
            return 3;                                                                   \
        }                                                                               \
    } while (0)

#define IO(cond)                                                \
    do {                                                        \
        if (!(cond)) {                                          \
            fprintf(stderr, "line %d: %s\n", __LINE__, #cond);  \
            return 4;                                           \
        }                                                       \
    } while (0)

typedef struct state_t {
    float *   theta, *m, *v, *gsum;
    uint16_t *tilde16, *theta16;
    int64_t   step, total;
} state_t;

static int alloc_state(state_t* s, int64_t n, const float* h_theta, const float* h_m, const float* h_v,
                       int64_t step0)
{
    size_t b4 = (size_t)n * 4, b2 = (size_t)n * 2;
    HIP(hipMalloc((void**)&s->theta, b4));
    HIP(hipMalloc((void**)&s->m, b4));
    HIP(hipMalloc((void**)&s->v, b4));
    HIP(hipMalloc((void**)&s->gsum, b4));
    HIP(hipMalloc((void**)&s->tilde16, b2));
    HIP(hipMalloc((void**)&s->theta16, b2));
    HIP(hipMemcpy(s->theta, h_theta, b4, hipMemcpyHostToDevice));
    HIP(hipMemcpy(s->m, h_m, b4, hipMemcpyHostToDevice));
    HIP(hipMemcpy(s->v, h_v, b4, hipMemcpyHostToDevice));
    HIP(hipMemset(s->gsum, 0xff, b4)); /* NaNs: stage 1 must overwrite, not add */
    HIP(hipMemset(s->tilde16, 0, b2));
    HIP(hipMemset(s->theta16, 0, b2));
    s->step  = step0;
    s->total = 0;
    return 0;
}

static int write_state(FILE* f, const state_t* s, int64_t n, void* host)
{
    size_t b4 = (size_t)n * 4, b2 = (size_t)n * 2;
    const void* arr[5];
    size_t      len[5];
    int         i;
    arr[0] = s->tilde16; len[0] = b2;
    arr[1] = s->theta;   len[1] = b4;
    arr[2] = s->m;       len[2] = b4;
    arr[3] = s->v;       len[3] = b4;
    arr[4] = s->theta16; len[4] = b2;
    for (i = 0; i < 5; ++i) {
        HIP(hipMemcpy(host, arr[i], len[i], hipMemcpyDeviceToHost));
        IO(fwrite(host, 1, len[i], f) == len[i]);
    }
    IO(fwrite(&s->step, 8, 1, f) == 1);
    IO(fwrite(&s->total, 8, 1, f) == 1);
    return 0;
}

int main(int argc, char** argv)
{
    int64_t      hdr[4], n, W, K, counts[MAXW];
    double       hpd[5];
    acco_adamw_t hp;
    FILE *       in, *out;
    float *      h_theta, *h_m, *h_v, *acc[MAXW];
    uint16_t *   h_g, *grad[2][MAXW][MAXK], *comm[MAXW], *stash[MAXW];
    const void*  shards[MAXW];
    state_t      base, fused;
    hipStream_t  stream;
    int          stage, w, k, rc;
    size_t       b4, b2;

    if (argc != 3) {
        fprintf(stderr, "usage: %s IN OUT\n", argv[0]);
        return 1;
    }
    in = fopen(argv[1], "rb");
    IO(in != NULL);
    IO(fread(hdr, 8, 4, in) == 4);
    IO(fread(hpd, 8, 5, in) == 5);
    n = hdr[0]; W = hdr[1]; K = hdr[2];
    IO(n >= 1 && W >= 1 && W <= MAXW && K >= 1 && K <= MAXK);
    hp.lr = hpd[0]; hp.beta1 = hpd[1]; hp.beta2 = hpd[2]; hp.eps = hpd[3]; hp.weight_decay = hpd[4];
    b4 = (size_t)n * 4;
    b2 = (size_t)n * 2;
    h_theta = (float*)malloc(b4);
    h_m     = (float*)malloc(b4);
    h_v     = (float*)malloc(b4);
    h_g     = (uint16_t*)malloc(b4); /* also the staging buffer for the results */
    IO(h_theta && h_m && h_v && h_g);
    IO(fread(h_theta, 4, (size_t)n, in) == (size_t)n);
    IO(fread(h_m, 4, (size_t)n, in) == (size_t)n);
    IO(fread(h_v, 4, (size_t)n, in) == (size_t)n);

    HIP(hipSetDevice(0));
    HIP(hipStreamCreate(&stream));
    for (stage = 0; stage < 2; ++stage)
        for (w = 0; w < W; ++w)
            for (k = 0; k < K; ++k) {
                IO(fread(h_g, 2, (size_t)n, in) == (size_t)n);
                HIP(hipMalloc((void**)&grad[stage][w][k], b2));
                HIP(hipMemcpy(grad[stage][w][k], h_g, b2, hipMemcpyHostToDevice));
            }
    fclose(in);
    for (w = 0; w < W; ++w) {
        HIP(hipMalloc((void**)&acc[w], b4));
        HIP(hipMalloc((void**)&comm[w], b2));
        HIP(hipMalloc((void**)&stash[w], b2));
        shards[w] = comm[w];
    }
    if ((rc = alloc_state(&base, n, h_theta, h_m, h_v, hdr[3])) != 0) return rc;
    if ((rc = alloc_state(&fused, n, h_theta, h_m, h_v, hdr[3])) != 0) return rc;

    /* the five base entry points, one call per line of Alg. 1's communication stream */
    for (stage = 0; stage < 2; ++stage) {
        for (w = 0; w < W; ++w) {
            for (k = 0; k < K; ++k)
                ACCO(acco_accumulate(acc[w], grad[stage][w][k], n, k == 0, &counts[w], stream));
            ACCO(acco_cast_params(comm[w], acc[w], n, stream));
        }
        ACCO(acco_reduce_shards(base.gsum, shards, (int)W, ACCO_BF16, n, stage, counts, &base.total, NULL,
                                NULL, stream));
        if (stage == 0)
            ACCO(acco_estimate_step(base.theta, base.m, base.v, base.gsum, NULL, base.tilde16, n, &hp,
                                    base.step, base.total, NULL, stream));
        else
            ACCO(acco_commit_step(base.theta, base.m, base.v, base.gsum, base.theta16, n, &hp, &base.step,
                                  base.total, NULL, stream));
        for (w = 0; w < W; ++w) IO(counts[w] == K);
    }
    HIP(hipStreamSynchronize(stream));

    /* the fused forms: bf16 stash of the first micro-batch, publish fused into the last
     * accumulation, reduction fused into the step */
    for (stage = 0; stage < 2; ++stage) {
        for (w = 0; w < W; ++w) {
            HIP(hipMemsetAsync(comm[w], 0, b2, stream));
            if (K == 1) {
                ACCO(acco_accumulate_first(comm[w], grad[stage][w][0], n, 1, &counts[w], stream));
                continue;
            }
            ACCO(acco_accumulate_first(stash[w], grad[stage][w][0], n, 0, &counts[w], stream));
            if (K == 2) {
                ACCO(acco_accumulate_second(NULL, comm[w], stash[w], grad[stage][w][1], n, &counts[w],
                                            stream));
                continue;
            }
            ACCO(acco_accumulate_second(acc[w], NULL, stash[w], grad[stage][w][1], n, &counts[w], stream));
            for (k = 2; k + 1 < K; ++k)
                ACCO(acco_accumulate(acc[w], grad[stage][w][k], n, 0, &counts[w], stream));
            ACCO(acco_accumulate_publish(acc[w], grad[stage][w][K - 1], comm[w], n, 0, 0, &counts[w],
                                         stream));
        }
        for (w = 0; w < W; ++w) IO(counts[w] == K);
        if (stage == 0)
            ACCO(acco_reduce_estimate_step(fused.theta, fused.m, fused.v, fused.gsum, shards, (int)W,
                                           ACCO_BF16, counts, &fused.total, NULL, fused.tilde16, n, &hp,
                                           fused.step, NULL, NULL, stream));
        else
            ACCO(acco_reduce_commit_step(fused.theta, fused.m, fused.v, fused.gsum, shards, (int)W,
                                         ACCO_BF16, counts, &fused.total, fused.theta16, n, &hp,
                                         &fused.step, NULL, NULL, stream));
    }
    HIP(hipStreamSynchronize(stream));

    out = fopen(argv[2], "wb");
    IO(out != NULL);
    if ((rc = write_state(out, &base, n, h_g)) != 0) return rc;
    if ((rc = write_state(out, &fused, n, h_g)) != 0) return rc;
    IO(fclose(out) == 0);
    HIP(hipStreamDestroy(stream));
    printf("round_from_c ok: n=%lld W=%lld K=%lld step=%lld total=%lld\n", (long long)n, (long long)W,
           (long long)K, (long long)base.step, (long long)base.total);
    return 0;
}
