/* The header as a plain C translation unit, and the library called from C with no Python in
 * between: validation, host counters and the host-only helpers (no device work: n == 0). */
#include <stdio.h>
#include <string.h>

#include "acco.h"

#define CHECK(cond)                                                   \
    do {                                                              \
        if (!(cond)) {                                                \
            fprintf(stderr, "line %d: %s\n", __LINE__, #cond);        \
            return 1;                                                 \
        }                                                             \
    } while (0)

int main(void)
{
    acco_adamw_t        hp = {6e-4, 0.9, 0.95, 1e-8, 0.1};
    acco_step_scalars_t sc;
    int64_t             count = 0, total = 0, step = 0;
    int64_t             counts[2] = {3, 4};
    const void*         shards[2];
    char*               base = (char*)0x100000; /* aligned fake addresses: never dereferenced at n == 0 */
    float *             theta = (float*)base, *m = (float*)(base + 0x1000), *v = (float*)(base + 0x2000),
          *gsum = (float*)(base + 0x3000);

    shards[0] = base + 0x4000;
    shards[1] = base + 0x5000;
    CHECK(acco_version() >= 500);
    CHECK(strstr(acco_status_string(ACCO_ERR_ALIGN), "ALIGN") != NULL);
    CHECK(acco_accumulate(theta, (const uint16_t*)shards[0], 0, 1, &count, NULL) == ACCO_OK && count == 1);
    CHECK(acco_accumulate(theta, (const uint16_t*)shards[0], 0, 0, &count, NULL) == ACCO_OK && count == 2);
    CHECK(acco_accumulate(NULL, NULL, -1, 0, &count, NULL) == ACCO_ERR_SIZE && count == 2);
    CHECK(acco_reduce_shards(gsum, shards, 2, ACCO_BF16, 0, 0, counts, &total, NULL, NULL, NULL) == ACCO_OK);
    CHECK(total == 7);
    CHECK(acco_estimate_step(theta, m, v, gsum, NULL, (uint16_t*)shards[1], 0, &hp, step, total, NULL,
                             NULL) == ACCO_OK && step == 0);
    CHECK(acco_reduce_shards(gsum, shards, 2, ACCO_BF16, 0, 1, counts, &total, NULL, NULL, NULL) == ACCO_OK);
    CHECK(total == 14);
    CHECK(acco_commit_step(theta, m, v, gsum, (uint16_t*)shards[1], 0, &hp, &step, total, NULL, NULL) ==
          ACCO_OK);
    CHECK(step == 1);
    CHECK(acco_commit_step(theta, theta, v, gsum, NULL, 8, &hp, &step, total, NULL, NULL) == ACCO_ERR_ALIAS);
    CHECK(step == 1);
    CHECK(acco_fold_adamw(&hp, step, total, &sc) == ACCO_OK);
    CHECK(sc.f[0] == (float)(1.0 / 14.0) && sc.f[1] == 0.9f && sc.f[2] == 0.95f);
    CHECK(acco_commit_step_resident(theta, m, v, gsum, NULL, 0, &sc, ACCO_RESIDENT_SLOTS, NULL, NULL) ==
          ACCO_ERR_SIZE);
    CHECK(acco_lr_cosine(6e-4, 0.0, 0, 0, 50000) == 6e-4);
    CHECK(sizeof(acco_step_scalars_t) == 64 && sizeof(acco_layout_t) == 16);
    printf("acco C ABI ok, version %d\n", acco_version());
    return 0;
}
