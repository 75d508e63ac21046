/* Test-only driver: runs every oracle routine on small inputs so that an AddressSanitizer /
 * UndefinedBehaviorSanitizer build of marsit_oracle.c can report out-of-bounds accesses, overflows
 * and the like.  Built and run by tests/test_oracle_sanitizers.py; prints "ok" and exits 0. */
#include <stdio.h>
#include <stdlib.h>
#include <stdint.h>

#include "../../oracle/marsit_oracle.c"

static float frand(uint64_t *state)
{
    *state = *state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((int64_t)(*state >> 40) - (1 << 23)) / (float)(1 << 23);
}

static int run_case(uint32_t M, uint64_t d, uint64_t ld, uint32_t grid_x)
{
    uint64_t W = (d + 63) / 64, state = 1234 + M * 31 + d;
    float *g = malloc(sizeof(float) * M * ld), *c = malloc(sizeof(float) * M * ld);
    float *update = malloc(sizeof(float) * (d ? d : 1));
    uint64_t *bits = malloc(sizeof(uint64_t) * (W ? W : 1)), *maps = malloc(sizeof(uint64_t) * (M * W ? M * W : 1));
    uint64_t *ref = malloc(sizeof(uint64_t) * (W ? W : 1));
    float *norms = malloc(sizeof(float) * M);
    if (!g || !c || !update || !bits || !maps || !ref || !norms)
        return 1;
    for (uint64_t i = 0; i < M * ld; ++i) {
        g[i] = frand(&state);
        c[i] = 0.25f * frand(&state);
    }
    int rc = 0;
    rc |= oracle_sync_step(g, c, update, bits, maps, M, d, ld, 1e-3f, 42, grid_x, 1);
    rc |= oracle_sync_step(g, c, update, bits, NULL, M, d, ld, 1e-3f, 43, grid_x, 2);
    rc |= oracle_ragged_torus_step(g, c, update, bits, M, d, ld, 1e-3f, 46, (M > 2) ? M - 1 : 1, 2);
    if (grid_x == 0) {
        rc |= oracle_tree_step(g, c, update, bits, M, d, ld, 1e-3f, 44);
        rc |= oracle_cascade_ring_step(g, c, update, bits, norms, M, d, ld, 45);
    }
    oracle_aggregate_sign(g, c, ref, M, d, ld);
    oracle_majority_vote(g, c, bits, M, d, ld);
    (void)oracle_count_matching(bits, ref, d);
    rc |= oracle_full_sync(g, c, update, M, d, ld);
    rc |= oracle_local_momentum(c, g, g, M, d, ld, 0.9f, 0.1f);
    if (d > 0)
        oracle_apply_update(g, update, d);
    free(g); free(c); free(update); free(bits); free(maps); free(ref); free(norms);
    return rc;
}

int main(void)
{
    int rc = 0;
    rc |= run_case(1, 1, 1, 0);
    rc |= run_case(2, 63, 64, 0);
    rc |= run_case(3, 65, 65, 0);
    rc |= run_case(8, 64 * 5 + 7, 64 * 5 + 9, 0);
    rc |= run_case(64, 100, 100, 0);          /* more workers than packed words */
    rc |= run_case(6, 1000, 1003, 3);
    rc |= run_case(16, 4097, 4097, 4);
    rc |= run_case(12, 129, 130, 2);
    rc |= run_case(5, 0, 4, 0);               /* empty input */
    uint64_t recv[3] = {1, 2, 3}, local[3] = {~0ULL, 0, 5}, out[3];
    rc |= oracle_hop_merge(recv, local, out, (1ULL << 40) + 3, 3, 1, 0, 7);
    rc |= oracle_hop_merge(recv, local, out, 0, 3, 64, 63, 7);
    rc |= oracle_hop_merge_weighted(recv, local, out, 0, 3, 0, 1, 5, 7);
    rc |= oracle_hop_merge_weighted(recv, local, out, 0, 3, 63, 1, 5, 7);
    if (rc != 0) {
        printf("oracle routine returned an error: %d\n", rc);
        return 1;
    }
    printf("ok\n");
    return 0;
}
