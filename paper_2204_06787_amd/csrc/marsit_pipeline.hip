// The one-bit pass as a ring of M workers that each own a HIP stream: every hop is its own launch
// and waits only for what a real ring would wait for (the segment arriving from the previous
// worker, and the previous use of its send buffer being consumed).  On one GPU the "transport" is
// an event plus a buffer that the next worker reads; with one worker per GPU the same graph has a
// peer copy where the event is.  Nothing here computes: it sequences marsit_compress,
// marsit_hop_merge and marsit_decode_compensate.
//
// Schedule (Section 4 of the paper, Fig. 3's reduce period): part i starts at worker i; at hop step
// h = 1..M-1 worker w folds its own signs of part (w - h) mod M into what worker w-1 sent.  A worker
// computes the signs of a part right before it needs them, so sign computation overlaps the wait
// for the incoming segment (Algorithm 1: receive in parallel with the sign step).  The gather period is a no-op here: the last
// holder writes the final segment where every worker reads it.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <new>

#include "marsit.h"

struct marsit_pipeline {
    uint32_t M;
    int device;
    hipStream_t worker[MARSIT_MAX_WORKERS];
    hipEvent_t start;
    hipEvent_t done[MARSIT_MAX_WORKERS];
    hipEvent_t hop[MARSIT_MAX_WORKERS][MARSIT_MAX_WORKERS];   // [hop step][worker]
};

namespace {

thread_local int tls_pipeline_hip_error = 0;

bool ok(hipError_t e)
{
    if (e == hipSuccess)
        return true;
    tls_pipeline_hip_error = static_cast<int>(e);
    return false;
}

void destroy_objects(marsit_pipeline *p)
{
    for (uint32_t w = 0; w < p->M; ++w) {
        if (p->worker[w] != nullptr)
            (void)hipStreamDestroy(p->worker[w]);
        if (p->done[w] != nullptr)
            (void)hipEventDestroy(p->done[w]);
        for (uint32_t h = 0; h < p->M; ++h)
            if (p->hop[h][w] != nullptr)
                (void)hipEventDestroy(p->hop[h][w]);
    }
    if (p->start != nullptr)
        (void)hipEventDestroy(p->start);
}

}   // namespace

extern "C" {

int marsit_pipeline_last_hip_error(void) { return tls_pipeline_hip_error; }

int marsit_pipeline_create(marsit_pipeline **out, uint32_t M)
{
    if (out == nullptr || M == 0 || M > MARSIT_MAX_WORKERS)
        return MARSIT_EINVAL;
    marsit_pipeline *p = new (std::nothrow) marsit_pipeline();
    if (p == nullptr)
        return MARSIT_EINVAL;
    p->M = M;
    bool good = ok(hipGetDevice(&p->device));
    // default priority on purpose; non-blocking so the workers do not serialise on the NULL stream
    for (uint32_t w = 0; good && w < M; ++w)
        good = ok(hipStreamCreateWithFlags(&p->worker[w], hipStreamNonBlocking)) &&
               ok(hipEventCreateWithFlags(&p->done[w], hipEventDisableTiming));
    good = good && ok(hipEventCreateWithFlags(&p->start, hipEventDisableTiming));
    for (uint32_t h = 0; good && h < M; ++h)
        for (uint32_t w = 0; good && w < M; ++w)
            good = ok(hipEventCreateWithFlags(&p->hop[h][w], hipEventDisableTiming));
    if (!good) {
        destroy_objects(p);
        delete p;
        return MARSIT_EHIP;
    }
    *out = p;
    return MARSIT_OK;
}

int marsit_pipeline_destroy(marsit_pipeline *p)
{
    if (p == nullptr)
        return MARSIT_EINVAL;
    bool good = true;
    for (uint32_t w = 0; w < p->M; ++w)
        good = ok(hipStreamSynchronize(p->worker[w])) && good;
    destroy_objects(p);
    delete p;
    return good ? MARSIT_OK : MARSIT_EHIP;
}

uint64_t marsit_pipeline_workspace_words(uint32_t M, uint64_t d)
{
    if (M == 0 || M > MARSIT_MAX_WORKERS || d > (static_cast<uint64_t>(1) << 37))
        return 0;
    const uint64_t W = (d + 63) / 64;
    const uint64_t part_max = W / M + 1;
    return static_cast<uint64_t>(M) * W + 2u * M * part_max;
}

int marsit_pipeline_ring_step(marsit_pipeline *p, const float *g, float *c, float *update_out,
                              uint64_t *bits_out, uint64_t *workspace, uint64_t d, uint64_t ld,
                              float scale, uint64_t seed, void *stream)
{
    if (p == nullptr || g == nullptr || c == nullptr || update_out == nullptr || bits_out == nullptr ||
        workspace == nullptr || ld < d || !std::isfinite(scale) ||
        d > (static_cast<uint64_t>(1) << 37))
        return MARSIT_EINVAL;
    if (reinterpret_cast<uintptr_t>(g) % 4 || reinterpret_cast<uintptr_t>(c) % 4 ||
        reinterpret_cast<uintptr_t>(update_out) % 4 || reinterpret_cast<uintptr_t>(bits_out) % 8 ||
        reinterpret_cast<uintptr_t>(workspace) % 8)
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;

    const uint32_t M = p->M;
    const uint64_t W = (d + 63) / 64;
    const uint64_t part_max = W / M + 1;
    uint64_t bound[MARSIT_MAX_WORKERS + 1];
    int rc = marsit_split_bounds(W, M, 0, bound);
    if (rc != MARSIT_OK)
        return rc;
    uint64_t *maps = workspace;                                   // [M][W]   own signs
    uint64_t *seg = workspace + static_cast<size_t>(M) * W;       // [2][M][part_max]  send buffers
    hipStream_t caller = static_cast<hipStream_t>(stream);

    // signs of part i of worker w, written into the worker's own bitmap
    auto compress_part = [&](uint32_t w, uint32_t i) -> int {
        const uint64_t lo = bound[i], hi = bound[i + 1];
        if (hi == lo)
            return MARSIT_OK;
        const uint64_t e0 = lo * 64, e1 = (hi * 64 < d) ? hi * 64 : d;
        return marsit_compress(g + static_cast<size_t>(w) * ld + e0, c + static_cast<size_t>(w) * ld + e0,
                               maps + static_cast<size_t>(w) * W + lo, e1 - e0, p->worker[w]);
    };

    if (!ok(hipEventRecord(p->start, caller)))
        return MARSIT_EHIP;
    for (uint32_t w = 0; w < M; ++w)
        if (!ok(hipStreamWaitEvent(p->worker[w], p->start, 0)))
            return MARSIT_EHIP;

    // hop step 0: every worker computes the signs of the part it starts and "sends" them
    for (uint32_t w = 0; w < M; ++w) {
        rc = compress_part(w, w);
        if (rc != MARSIT_OK)
            return rc;
        if (M == 1 && bound[1] > bound[0]) {
            // a single worker: its own signs are the final bitmap (fold 1 copies them)
            rc = marsit_hop_merge(maps, maps, bits_out, 0, W, 1, 0, seed, p->worker[0]);
            if (rc != MARSIT_OK)
                return rc;
        }
        if (!ok(hipEventRecord(p->hop[0][w], p->worker[w])))
            return MARSIT_EHIP;
    }

    // hop steps 1..M-1 (the reduce period)
    for (uint32_t h = 1; h < M; ++h) {
        for (uint32_t w = 0; w < M; ++w) {
            const uint32_t i = (w + M - h % M) % M;          // the part that reaches worker w now
            const uint32_t prev = (w + M - 1) % M, next = (w + 1) % M;
            const uint64_t lo = bound[i], n = bound[i + 1] - lo;
            // own signs of that part: overlaps the wait for the incoming segment
            rc = compress_part(w, i);
            if (rc != MARSIT_OK)
                return rc;
            // the segment from the previous worker has arrived
            if (!ok(hipStreamWaitEvent(p->worker[w], p->hop[h - 1][prev], 0)))
                return MARSIT_EHIP;
            // this worker's send buffer of two hops ago has been consumed by the next worker
            if (h >= 3 && !ok(hipStreamWaitEvent(p->worker[w], p->hop[h - 1][next], 0)))
                return MARSIT_EHIP;
            if (n > 0) {
                const uint64_t *recv = (h == 1)
                    ? maps + static_cast<size_t>(prev) * W + lo
                    : seg + (static_cast<size_t>((h - 1) & 1u) * M + prev) * part_max;
                uint64_t *out = (h == M - 1)
                    ? bits_out + lo
                    : seg + (static_cast<size_t>(h & 1u) * M + w) * part_max;
                rc = marsit_hop_merge(recv, maps + static_cast<size_t>(w) * W + lo, out, lo, n, h + 1, h,
                                      seed, p->worker[w]);
                if (rc != MARSIT_OK)
                    return rc;
            }
            if (!ok(hipEventRecord(p->hop[h][w], p->worker[w])))
                return MARSIT_EHIP;
        }
    }

    // gather period (simulated): every worker waits until all final parts exist, then decodes
    for (uint32_t w = 0; w < M; ++w) {
        for (uint32_t v = 0; v < M; ++v)
            if (v != w && !ok(hipStreamWaitEvent(p->worker[w], p->hop[M - 1][v], 0)))
                return MARSIT_EHIP;
        rc = marsit_decode_compensate(bits_out, g + static_cast<size_t>(w) * ld,
                                      c + static_cast<size_t>(w) * ld, scale,
                                      w == 0 ? update_out : nullptr, c + static_cast<size_t>(w) * ld, d,
                                      p->worker[w]);
        if (rc != MARSIT_OK)
            return rc;
        if (!ok(hipEventRecord(p->done[w], p->worker[w])) ||
            !ok(hipStreamWaitEvent(caller, p->done[w], 0)))
            return MARSIT_EHIP;
    }
    return MARSIT_OK;
}

}   // extern "C"
