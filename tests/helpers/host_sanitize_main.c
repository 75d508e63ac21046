/*
 * Host-side logic of libmarsit under AddressSanitizer / UndefinedBehaviorSanitizer: every call below
 * returns before anything is enqueued on a GPU (host utilities, size arithmetic, argument
 * validation), so the program runs on a machine without one.  Prints "ok" at the end.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "marsit.h"

#define CHECK(cond)                                                            \
    do {                                                                       \
        if (!(cond)) {                                                         \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                          \
        }                                                                      \
    } while (0)

static void *fake(uintptr_t offset) { return (void *)(uintptr_t)(0x10000000u + offset); }

int main(void)
{
    /* split bounds: floor rule, monotone, ends at n_words, for every worker count and grid */
    static const uint64_t sizes[] = {0, 1, 2, 63, 64, 65, 400000, 0xFFFFFFFFull, (1ull << 28) - 16};
    for (size_t s = 0; s < sizeof sizes / sizeof sizes[0]; ++s) {
        for (uint32_t M = 1; M <= MARSIT_MAX_WORKERS; ++M) {
            for (uint32_t grid_x = 0; grid_x <= M; ++grid_x) {
                uint64_t bounds[MARSIT_MAX_WORKERS + 1];
                const int rc = marsit_split_bounds(sizes[s], M, grid_x, bounds);
                if (grid_x != 0 && M % grid_x != 0) {
                    CHECK(rc == MARSIT_EINVAL);
                    continue;
                }
                CHECK(rc == MARSIT_OK);
                CHECK(bounds[0] == 0 && bounds[M] == sizes[s]);
                for (uint32_t k = 0; k < M; ++k)
                    CHECK(bounds[k] <= bounds[k + 1]);
            }
        }
    }
    CHECK(marsit_split_bounds(10, 0, 0, NULL) == MARSIT_EINVAL);
    CHECK(marsit_split_bounds(10, MARSIT_MAX_WORKERS + 1, 0, NULL) == MARSIT_EINVAL);

    /* workspace and launch-width arithmetic at the extremes */
    for (uint32_t M = 1; M <= MARSIT_MAX_WORKERS; ++M) {
        CHECK(marsit_chain_workspace_words(M, 0, 0) == 0 || marsit_chain_workspace_words(M, 0, 0) > 0);
        const uint64_t w = marsit_chain_workspace_words(M, MARSIT_MAX_ELEMENTS, 0);
        CHECK(w >= (MARSIT_MAX_ELEMENTS / 64) * (uint64_t)M);
        CHECK(marsit_pipeline_workspace_words(M, MARSIT_MAX_ELEMENTS, 0) >= w / 2);
    }
    CHECK(marsit_grid_work_items(0) == 0);
    CHECK(marsit_grid_work_items(1) == 256);
    CHECK(marsit_grid_work_items(MARSIT_MAX_ELEMENTS) < (1ull << 32));
    CHECK(marsit_grid_work_items(MARSIT_MAX_ELEMENTS + 1) == 0);

    /* host Philox: known answer of the published generator for the all-zero input */
    const uint32_t ctr[4] = {0, 0, 0, 0}, key[2] = {0, 0};
    uint32_t out[4];
    marsit_philox4x32_10(ctr, key, out);
    CHECK(out[0] == 0x6627e8d5u && out[1] == 0xe169c58du && out[2] == 0xbc57ac4cu && out[3] == 0x9b00dbd8u);

    /* status strings for every code and for codes that do not exist */
    for (int code = -10; code <= 2; ++code)
        CHECK(marsit_status_string(code) != NULL);
    CHECK(marsit_version() >= 100);

    /* argument validation: each call must be turned away before any launch */
    float *g = fake(0), *c = fake(1 << 20), *u = fake(2 << 20), *x = fake(3 << 20);
    uint64_t *b = fake(4 << 20), *ws = fake(5 << 20);
    CHECK(marsit_ring_step_sim(NULL, c, u, b, 8, 64, 64, 1.0f, 1, 0, NULL) == MARSIT_EINVAL);
    CHECK(marsit_ring_step_sim(g, c, u, b, 0, 64, 64, 1.0f, 1, 0, NULL) == MARSIT_EINVAL);
    CHECK(marsit_ring_step_sim(g, c, u, b, MARSIT_MAX_WORKERS + 1, 64, 64, 1.0f, 1, 0, NULL) == MARSIT_EINVAL);
    CHECK(marsit_ring_step_sim(g, c, u, b, 8, 64, 32, 1.0f, 1, 0, NULL) == MARSIT_EINVAL);
    CHECK(marsit_ring_step_sim(g, c, u, b, 8, 64, 64, 1.0f, 1, 3, NULL) == MARSIT_EINVAL);
    CHECK(marsit_ring_step_sim(g, c, u, b, 8, MARSIT_MAX_ELEMENTS + 1, MARSIT_MAX_ELEMENTS + 1, 1.0f, 1, 0, NULL) ==
          MARSIT_EINVAL);
    CHECK(marsit_ring_step_sim((float *)((char *)g + 2), c, u, b, 8, 64, 64, 1.0f, 1, 0, NULL) == MARSIT_EALIGN);
    CHECK(marsit_ring_step_sim(g, c, u, b, 8, 0, 64, 1.0f, 1, 0, NULL) == MARSIT_OK);
    CHECK(marsit_round(1, 0, MARSIT_SCHEDULE_RING, 0, g, c, x, u, b, 8, 64, 64, 1.0f, 1, NULL) == MARSIT_EINVAL);
    CHECK(marsit_round(1, 4, 99, 0, g, c, x, u, b, 8, 64, 64, 1.0f, 1, NULL) == MARSIT_EINVAL);
    CHECK(marsit_round(1, 4, MARSIT_SCHEDULE_TORUS, 0, g, c, x, u, b, 8, 64, 64, 1.0f, 1, NULL) == MARSIT_EINVAL);
    CHECK(marsit_round(1, 4, MARSIT_SCHEDULE_TREE, 0, g, c, x, u, b, 8, 0, 64, 1.0f, 1, NULL) == MARSIT_OK);
    CHECK(marsit_full_sync(g, c, NULL, 8, 64, 64, NULL) == MARSIT_EINVAL);
    CHECK(marsit_tree_step_sim(g, c, u, b, 65, 64, 64, 1.0f, 1, NULL) == MARSIT_EINVAL);
    CHECK(marsit_ragged_torus_step_sim(g, c, u, b, 13, 64, 64, 1.0f, 1, 14, NULL) == MARSIT_EINVAL);
    CHECK(marsit_exchange_step_sim(g, c, u, b, NULL, 8, 64, 64, 1.0f, 1, 0, NULL) == MARSIT_EINVAL);
    CHECK(marsit_exchange_step_sim_static(g, c, u, b, 8, MARSIT_MAX_ELEMENTS, MARSIT_MAX_ELEMENTS, 1.0f, 1, 0, NULL) ==
          MARSIT_ESCRATCH);
    CHECK(marsit_chain_step_sim(g, c, u, b, ws, 8, 64, 32, 1.0f, 1, 0, NULL) == MARSIT_EINVAL);
    CHECK(marsit_compress(g, c, NULL, 64, NULL) == MARSIT_EINVAL);
    CHECK(marsit_hop_merge(b, b + 8, b + 16, 0, 4, 0, 1, 1, NULL) == MARSIT_EINVAL);
    CHECK(marsit_decode_compensate(b, g, c, 1.0f, u, NULL, 64, NULL) == MARSIT_EINVAL);
    CHECK(marsit_local_momentum(g, g, u, 2, 64, 64, 0.9f, 0.1f, NULL) == MARSIT_EINVAL);
    CHECK(marsit_local_adam(g, c, u, x, 2, 64, 64, 0.9f, 0.999f, 1e-8f, 0.1f, 0.0f, 0.1f, NULL) == MARSIT_EINVAL);
    CHECK(marsit_set_fused_waves_per_cu(1) == MARSIT_EINVAL);
    CHECK(marsit_set_fused_waves_per_cu(33) == MARSIT_EINVAL);
    CHECK(marsit_set_fused_waves_per_cu(0) == MARSIT_OK);
    puts("ok");
    return 0;
}
