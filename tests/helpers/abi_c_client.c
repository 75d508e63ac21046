/* Test-only client of the C ABI written in plain C (no C++, no Python, no torch): reads a small
 * problem from a file, allocates device memory with the HIP runtime, runs the fused pass through
 * marsit_ring_step_sim for the given number of steps and writes the results to a file.  Built by
 * paper_2204_06787_amd/build.py with gcc; tests/test_gpu_c_client.py feeds it seeded inputs and
 * compares what it writes with the CPU oracle.
 *
 * Input file:  u32 M, u32 grid_x, u64 d, u64 ld, f32 scale, u32 steps, u64 seed0, then
 *              steps * M * ld floats (the gradients of every step); compensation starts at zero;
 *              step t uses seed0 + t.
 * Output file: d floats (last update), ceil(d/64) u64 (last merged bitmap), M * ld floats (c).
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "marsit.h"

#define CHECK_HIP(call)                                                                  \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess) {                                                          \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));            \
            return 3;                                                                    \
        }                                                                                \
    } while (0)

static int read_exact(FILE *f, void *p, size_t n) { return fread(p, 1, n, f) == n ? 0 : -1; }

int main(int argc, char **argv)
{
    if (argc != 3) {
        fprintf(stderr, "usage: %s <input> <output>\n", argv[0]);
        return 2;
    }
    FILE *in = fopen(argv[1], "rb");
    if (!in) {
        perror("input");
        return 2;
    }
    uint32_t M, grid_x, steps;
    uint64_t d, ld, seed0;
    float scale;
    if (read_exact(in, &M, 4) || read_exact(in, &grid_x, 4) || read_exact(in, &d, 8) ||
        read_exact(in, &ld, 8) || read_exact(in, &scale, 4) || read_exact(in, &steps, 4) ||
        read_exact(in, &seed0, 8)) {
        fprintf(stderr, "short header\n");
        return 2;
    }
    const size_t n = (size_t)M * ld, W = (size_t)((d + 63) / 64);
    float *g_host = malloc(sizeof(float) * n * steps);
    float *c_host = malloc(sizeof(float) * n);
    float *u_host = malloc(sizeof(float) * (d ? d : 1));
    uint64_t *b_host = malloc(sizeof(uint64_t) * (W ? W : 1));
    if (!g_host || !c_host || !u_host || !b_host || read_exact(in, g_host, sizeof(float) * n * steps)) {
        fprintf(stderr, "cannot read %zu gradient values\n", n * steps);
        return 2;
    }
    fclose(in);

    float *g_dev, *c_dev, *u_dev;
    uint64_t *b_dev;
    hipStream_t stream;
    CHECK_HIP(hipSetDevice(0));
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_HIP(hipMalloc((void **)&g_dev, sizeof(float) * n));
    CHECK_HIP(hipMalloc((void **)&c_dev, sizeof(float) * n));
    CHECK_HIP(hipMalloc((void **)&u_dev, sizeof(float) * (d ? d : 1)));
    CHECK_HIP(hipMalloc((void **)&b_dev, sizeof(uint64_t) * (W ? W : 1)));
    memset(c_host, 0, sizeof(float) * n);
    CHECK_HIP(hipMemcpy(c_dev, c_host, sizeof(float) * n, hipMemcpyHostToDevice));

    printf("marsit_version %d, M=%u grid_x=%u d=%llu ld=%llu steps=%u\n", marsit_version(), M, grid_x,
           (unsigned long long)d, (unsigned long long)ld, steps);
    for (uint32_t t = 0; t < steps; ++t) {
        CHECK_HIP(hipMemcpy(g_dev, g_host + (size_t)t * n, sizeof(float) * n, hipMemcpyHostToDevice));
        const int rc = marsit_ring_step_sim(g_dev, c_dev, u_dev, b_dev, M, d, ld, scale, seed0 + t,
                                            grid_x, stream);
        if (rc != MARSIT_OK) {
            fprintf(stderr, "marsit_ring_step_sim: %s (hip error %d)\n", marsit_status_string(rc),
                    marsit_last_hip_error());
            return 4;
        }
        CHECK_HIP(hipStreamSynchronize(stream));
    }
    CHECK_HIP(hipMemcpy(u_host, u_dev, sizeof(float) * d, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(b_host, b_dev, sizeof(uint64_t) * W, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(c_host, c_dev, sizeof(float) * n, hipMemcpyDeviceToHost));

    FILE *out = fopen(argv[2], "wb");
    if (!out) {
        perror("output");
        return 2;
    }
    if (fwrite(u_host, sizeof(float), d, out) != d || fwrite(b_host, sizeof(uint64_t), W, out) != W ||
        fwrite(c_host, sizeof(float), n, out) != n) {
        fprintf(stderr, "short write\n");
        return 2;
    }
    fclose(out);
    CHECK_HIP(hipFree(g_dev));
    CHECK_HIP(hipFree(c_dev));
    CHECK_HIP(hipFree(u_dev));
    CHECK_HIP(hipFree(b_dev));
    CHECK_HIP(hipStreamDestroy(stream));
    free(g_host); free(c_host); free(u_host); free(b_host);
    printf("ok\n");
    return 0;
}
