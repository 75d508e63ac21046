// The one-bit pass as a ring of M workers that each own a HIP stream: every hop is its own launch
// and waits only for what a real ring would wait for (the segment arriving from the previous
// worker, and the previous use of its send buffer being consumed).  On one GPU the "transport" is
// an event plus a buffer that the next worker reads; with one worker per GPU the same graph has a
// peer copy where the event is.  Nothing here computes: it sequences marsit_compress,
// marsit_compress_hop_merge, marsit_hop_merge and marsit_decode_compensate.
//
// Schedule (Section 4 of the paper, Fig. 3's reduce period): part i starts at worker i; at hop step
// h = 1..M-1 worker w folds its own signs of part (w - h) mod M into what worker w-1 sent.  A worker
// computes the signs of the part it starts before anything arrives (Algorithm 1: the sign step runs
// in parallel with the receive); for every later part the sign step is fused into the merge
// (marsit_compress_hop_merge): one launch per hop, and the part's signs are never stored.  On this
// device a part's sign step is a few microseconds of HBM time, less than a launch.  The gather
// period is a no-op here: the last
// holder writes the final segment where every worker reads it.
//
// Torus (grid_x columns): every row runs that ring over its X workers on the X row-parts; the row
// result of row-part a ends at the worker in column (a + X - 1) mod X.  The Y workers of that column
// then run a ring over the Y sub-parts of row-part a, operands being the row results, and the last
// holder of a sub-part writes it to the final bitmap.

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
    hipEvent_t hop[MARSIT_MAX_WORKERS][MARSIT_MAX_WORKERS];    // row phase    [hop step][worker]
    hipEvent_t chop[MARSIT_MAX_WORKERS][MARSIT_MAX_WORKERS];   // column phase [hop step][worker]
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
        for (uint32_t h = 0; h < p->M; ++h) {
            if (p->hop[h][w] != nullptr)
                (void)hipEventDestroy(p->hop[h][w]);
            if (p->chop[h][w] != nullptr)
                (void)hipEventDestroy(p->chop[h][w]);
        }
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
            good = ok(hipEventCreateWithFlags(&p->hop[h][w], hipEventDisableTiming)) &&
                   ok(hipEventCreateWithFlags(&p->chop[h][w], hipEventDisableTiming));
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

// Workspace layout (64-bit words): own sign bitmaps [M][W]; row-phase send buffers [2][M][rp];
// row results [Y][W] (torus only); column-phase send buffers [2][M][sp] (torus only), where rp / sp
// bound the words of a row-part / sub-part.
struct PipelineLayout {
    uint32_t X, Y;
    uint64_t W, rp, sp, maps, seg, rowres, cseg, total;
};

static bool pipeline_layout(uint32_t M, uint64_t d, uint32_t grid_x, PipelineLayout *L)
{
    if (M == 0 || M > MARSIT_MAX_WORKERS || d > MARSIT_MAX_ELEMENTS)
        return false;
    L->X = (grid_x == 0) ? M : grid_x;
    if (L->X == 0 || M % L->X != 0)
        return false;
    L->Y = M / L->X;
    L->W = (d + 63) / 64;
    L->rp = L->W / L->X + 1;
    L->sp = L->rp / L->Y + 1;
    L->maps = 0;
    L->seg = L->maps + static_cast<uint64_t>(M) * L->W;
    L->rowres = L->seg + 2u * M * L->rp;
    L->cseg = L->rowres + (L->Y > 1 ? static_cast<uint64_t>(L->Y) * L->W : 0);
    L->total = L->cseg + (L->Y > 1 ? 2u * M * L->sp : 0);
    return true;
}

uint64_t marsit_pipeline_workspace_words(uint32_t M, uint64_t d, uint32_t grid_x)
{
    PipelineLayout L;
    return pipeline_layout(M, d, grid_x, &L) ? L.total : 0;
}

int marsit_pipeline_step(marsit_pipeline *p, const float *g, float *c, float *update_out,
                         uint64_t *bits_out, uint64_t *workspace, uint64_t d, uint64_t ld, float scale,
                         uint64_t seed, uint32_t grid_x, void *stream)
{
    PipelineLayout L;
    if (p == nullptr || g == nullptr || c == nullptr || update_out == nullptr || bits_out == nullptr ||
        workspace == nullptr || ld < d || !std::isfinite(scale) || !pipeline_layout(p->M, d, grid_x, &L))
        return MARSIT_EINVAL;
    if (reinterpret_cast<uintptr_t>(g) % 4 || reinterpret_cast<uintptr_t>(c) % 4 ||
        reinterpret_cast<uintptr_t>(update_out) % 4 || reinterpret_cast<uintptr_t>(bits_out) % 8 ||
        reinterpret_cast<uintptr_t>(workspace) % 8)
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;

    const uint32_t M = p->M, X = L.X, Y = L.Y;
    const uint64_t W = L.W;
    uint64_t fine[MARSIT_MAX_WORKERS + 1];      // fine[a*Y + b]: start of sub-part b of row-part a
    int rc = marsit_split_bounds(W, M, grid_x, fine);
    if (rc != MARSIT_OK)
        return rc;
    uint64_t *maps = workspace + L.maps;
    uint64_t *seg = workspace + L.seg;
    uint64_t *rowres = (Y > 1) ? workspace + L.rowres : bits_out;   // a ring's row result is the final bitmap
    uint64_t *cseg = workspace + L.cseg;
    hipStream_t caller = static_cast<hipStream_t>(stream);
    auto stream_of = [&](uint32_t y, uint32_t x) { return p->worker[y * X + x]; };

    // signs of row-part a of worker (y, x), written into the worker's own bitmap
    auto compress_part = [&](uint32_t y, uint32_t x, uint32_t a) -> int {
        const uint64_t lo = fine[a * Y], hi = fine[(a + 1) * Y];
        if (hi == lo)
            return MARSIT_OK;
        const uint32_t w = y * X + x;
        const uint64_t e0 = lo * 64, e1 = (hi * 64 < d) ? hi * 64 : d;
        return marsit_compress(g + static_cast<size_t>(w) * ld + e0, c + static_cast<size_t>(w) * ld + e0,
                               maps + static_cast<size_t>(w) * W + lo, e1 - e0, p->worker[w]);
    };

    if (!ok(hipEventRecord(p->start, caller)))
        return MARSIT_EHIP;
    for (uint32_t w = 0; w < M; ++w)
        if (!ok(hipStreamWaitEvent(p->worker[w], p->start, 0)))
            return MARSIT_EHIP;

    // ---- row phase: in every row a ring over its X workers (the reduce period of Fig. 3) ----------
    // hop step 0: worker (y, x) computes the signs of the row-part it starts (a = x) and "sends" them
    for (uint32_t y = 0; y < Y; ++y) {
        for (uint32_t x = 0; x < X; ++x) {
            rc = compress_part(y, x, x);
            if (rc != MARSIT_OK)
                return rc;
            if (X == 1 && W > 0) {
                // a row of one worker: its own signs are the row result (fold 1 copies them)
                const uint32_t w = y;
                rc = marsit_hop_merge(maps + static_cast<size_t>(w) * W, maps + static_cast<size_t>(w) * W,
                                      rowres + static_cast<size_t>(Y > 1 ? y : 0) * W, 0, W, 1, 0, seed,
                                      p->worker[w]);
                if (rc != MARSIT_OK)
                    return rc;
            }
            if (!ok(hipEventRecord(p->hop[0][y * X + x], stream_of(y, x))))
                return MARSIT_EHIP;
        }
    }
    for (uint32_t h = 1; h < X; ++h) {
        for (uint32_t y = 0; y < Y; ++y) {
            for (uint32_t x = 0; x < X; ++x) {
                const uint32_t w = y * X + x;
                const uint32_t a = (x + X - h) % X;                 // the row-part that reaches (y, x) now
                const uint32_t prev = y * X + (x + X - 1) % X, next = y * X + (x + 1) % X;
                const uint64_t lo = fine[a * Y], n = fine[(a + 1) * Y] - lo;
                // the segment from the previous worker of the row has arrived
                if (!ok(hipStreamWaitEvent(p->worker[w], p->hop[h - 1][prev], 0)))
                    return MARSIT_EHIP;
                // this worker's send buffer of two hops ago has been consumed by the next worker
                if (h >= 3 && !ok(hipStreamWaitEvent(p->worker[w], p->hop[h - 1][next], 0)))
                    return MARSIT_EHIP;
                if (n > 0) {
                    const uint64_t *recv = (h == 1)
                        ? maps + static_cast<size_t>(prev) * W + lo
                        : seg + (static_cast<size_t>((h - 1) & 1u) * M + prev) * L.rp;
                    uint64_t *out = (h == X - 1)
                        ? rowres + static_cast<size_t>(Y > 1 ? y : 0) * W + lo
                        : seg + (static_cast<size_t>(h & 1u) * M + w) * L.rp;
                    // own signs of that part, computed in the same pass that folds them in
                    const uint64_t e0 = lo * 64, e1 = ((lo + n) * 64 < d) ? (lo + n) * 64 : d;
                    rc = marsit_compress_hop_merge(recv, g + static_cast<size_t>(w) * ld + e0,
                                                   c + static_cast<size_t>(w) * ld + e0, out, lo, e1 - e0,
                                                   h + 1, (y << 8) | h, seed, p->worker[w]);
                    if (rc != MARSIT_OK)
                        return rc;
                }
                if (!ok(hipEventRecord(p->hop[h][w], p->worker[w])))
                    return MARSIT_EHIP;
            }
        }
    }

    // ---- column phase (torus): the last holders of row-part a sit in column xs = (a + X - 1) mod X;
    // these Y workers run a ring over the Y sub-parts of row-part a, on the row results -----------
    const hipEvent_t *last = p->hop[X - 1];          // "row result of this worker's row-part is ready"
    if (Y > 1) {
        for (uint32_t k = 1; k < Y; ++k) {
            for (uint32_t a = 0; a < X; ++a) {
                const uint32_t xs = (a + X - 1) % X;
                for (uint32_t y = 0; y < Y; ++y) {
                    const uint32_t w = y * X + xs;
                    const uint32_t b = (y + Y - k) % Y;             // the sub-part that reaches row y now
                    const uint32_t prev = ((y + Y - 1) % Y) * X + xs, next = ((y + 1) % Y) * X + xs;
                    const uint64_t lo = fine[a * Y + b], n = fine[a * Y + b + 1] - lo;
                    const hipEvent_t *before = (k == 1) ? last : p->chop[k - 1];
                    if (!ok(hipStreamWaitEvent(p->worker[w], before[prev], 0)))
                        return MARSIT_EHIP;
                    if (k >= 3 && !ok(hipStreamWaitEvent(p->worker[w], p->chop[k - 1][next], 0)))
                        return MARSIT_EHIP;
                    if (n > 0) {
                        const uint64_t *recv = (k == 1)
                            ? rowres + static_cast<size_t>((y + Y - 1) % Y) * W + lo
                            : cseg + (static_cast<size_t>((k - 1) & 1u) * M + prev) * L.sp;
                        uint64_t *out = (k == Y - 1)
                            ? bits_out + lo
                            : cseg + (static_cast<size_t>(k & 1u) * M + w) * L.sp;
                        rc = marsit_hop_merge(recv, rowres + static_cast<size_t>(y) * W + lo, out, lo, n,
                                              k + 1, (1u << 16) | k, seed, p->worker[w]);
                        if (rc != MARSIT_OK)
                            return rc;
                    }
                    if (!ok(hipEventRecord(p->chop[k][w], p->worker[w])))
                        return MARSIT_EHIP;
                }
            }
        }
        last = p->chop[Y - 1];
    }

    // ---- gather period (simulated): every worker waits until all final parts exist, then decodes --
    for (uint32_t w = 0; w < M; ++w) {
        for (uint32_t v = 0; v < M; ++v)
            if (v != w && !ok(hipStreamWaitEvent(p->worker[w], last[v], 0)))
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

int marsit_pipeline_ring_step(marsit_pipeline *p, const float *g, float *c, float *update_out,
                              uint64_t *bits_out, uint64_t *workspace, uint64_t d, uint64_t ld,
                              float scale, uint64_t seed, void *stream)
{
    return marsit_pipeline_step(p, g, c, update_out, bits_out, workspace, d, ld, scale, seed, 0, stream);
}

}   // extern "C"
