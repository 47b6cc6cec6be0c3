/*
 * A plain C99 client of the library's C ABI: includes the public header, fills the configuration
 * struct, and walks the state machine of a round on a dry-run context (no GPU call is made, so it
 * runs anywhere the library loads).  Built and run by tests/test_abi_host.py; exit status 0 = pass.
 */
#include "cocod.h"

#include <stdio.h>
#include <string.h>

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); return 1; } \
    } while (0)

int main(void)
{
    const uint32_t W = 3;
    const uint64_t sizes[3] = { 5, 2000, 3 };
    uint64_t padded = 0, offsets[3], begins[4];
    uint32_t n_buckets = 0;
    CHECK(cocod_plan_layout(2008, 3, sizes, 0, &padded, offsets, &n_buckets, begins) == COCOD_OK);
    CHECK(offsets[0] == 0 && offsets[1] == 1024 && offsets[2] == 3072 && padded == 3076 && n_buckets == 1);

    cocod_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.struct_size = (uint32_t)sizeof cfg;
    cfg.W = W;
    cfg.d = 2008;
    cfg.n_tensors = 3;
    cfg.tensor_numel = sizes;
    cfg.grad = COCOD_GRAD_QUADRATIC;
    cfg.lr = 0.1f;
    cfg.momentum = 0.9f;
    cfg.stride = padded;
    /* dry run: the pointers are validated (non-null, aligned, disjoint) but never dereferenced */
    const uintptr_t base = 0x10000000u, big = (uintptr_t)W * padded * sizeof(float);
    cfg.xA = (float *)(base);
    cfg.xB = (float *)(base + big);
    cfg.v = (float *)(base + 2 * big);
    cfg.h = (const float *)(base + 3 * big);
    cfg.c = (const float *)(base + 4 * big);
    cfg.mean = (float *)(base + 5 * big);
    cfg.flags = COCOD_FLAG_DRY_RUN;

    cocod_ctx *ctx = NULL;
    CHECK(cocod_create(&cfg, &ctx) == COCOD_OK && ctx != NULL);
    uint64_t step = 99, pd = 0;
    uint32_t chunks = 0, buckets = 0;
    float *live = NULL;
    CHECK(cocod_get_plan(ctx, &pd, &chunks, &buckets) == COCOD_OK && pd == padded && chunks == 4 && buckets == 1);
    CHECK(cocod_average_end_apply(ctx) == COCOD_ERR_STATE);
    CHECK(strstr(cocod_last_error(ctx), "no round is open") != NULL);
    CHECK(cocod_average_begin(ctx) == COCOD_OK && cocod_is_averaging(ctx) == 1);
    CHECK(cocod_local_steps(ctx, 2) == COCOD_OK);
    CHECK(cocod_live_model(ctx, &live) == COCOD_OK && live == cfg.xB);
    CHECK(cocod_average_end_apply(ctx) == COCOD_OK && cocod_is_averaging(ctx) == 0);
    CHECK(cocod_average_begin(ctx) == COCOD_OK && cocod_local_steps_end_apply(ctx, 3) == COCOD_OK);
    CHECK(cocod_graph_round(ctx, 2, 1) == COCOD_ERR_INVALID);       /* the null stream cannot be captured */
    CHECK(cocod_average_begin(ctx) == COCOD_OK && cocod_local_steps(ctx, 2) == COCOD_OK);
    CHECK(cocod_average_apply_fused(ctx) == COCOD_OK && cocod_is_averaging(ctx) == 0);   /* closes the round */
    CHECK(cocod_average_apply_fused(ctx) == COCOD_OK && cocod_is_averaging(ctx) == 0);   /* blocking average while idle */
    CHECK(cocod_get_step(ctx, &step) == COCOD_OK && step == 7);
    CHECK(cocod_set_schedule(ctx, COCOD_SCHED_HEAD) == COCOD_OK && cocod_set_schedule(ctx, 17) == COCOD_ERR_INVALID);
    CHECK(cocod_local_steps(ctx, -1) == COCOD_ERR_INVALID);
    CHECK(cocod_destroy(ctx) == COCOD_OK);

    cfg.struct_size -= 4;                       /* a caller built against another header is refused */
    CHECK(cocod_create(&cfg, &ctx) == COCOD_ERR_INVALID && ctx == NULL);
    CHECK(cocod_version() >= 1000);
    puts("c abi client: ok");
    return 0;
}
