// Fused kernels of the Marsit one-bit synchronisation pass (gfx950) and their entry points.
//
// The operation is the one-bit branch of Algorithm 1 of the paper (mod(t,K) != 0) with the
// transient vector of Eq. 2 and the merge operator of Section 4.1.1.  The merge
//     (r AND l) OR ((r XOR l) AND v),  v = XNOR(l, t),  t ~ Bernoulli(1/m)
// reduces, bit by bit, to "t ? l : r" (check the eight cases), so a chain of merges is carried
// here as a running selection: after the chain, every bit is the sign bit of the worker picked by
// the last successful draw.  The selection is done on the fp32 words themselves; only bit 31 of
// the result is ever looked at.
//
// Everything is bandwidth-bound elementwise and bit work: 128-bit coalesced accesses, the random
// draws generated in registers, LDS only as a staging area of the generic kernels, no matrix cores.

#include "marsit_device.hpp"
#include "marsit_host.hpp"

#include <atomic>

namespace marsit {

// Bounds of the M parts of the packed words (word indices), passed by value in the kernel
// arguments so that a compile-time index becomes a scalar load.
struct PartTable {
    uint32_t bound[MARSIT_MAX_WORKERS + 1];
    uint32_t xcd_group;     // compiled schedules, rows off the 128-byte lines: tiles per XCD run
};

// Keep thresholds floor(2^32 / fold) for the kernels whose fold counts are run-time values.
struct ThresholdTable {
    uint32_t thr[MARSIT_MAX_WORKERS + 1];
};

// -------------------------------------------------------------------------------------------------
// Fused pass, schedule known at compile time: X columns, Y rows (ring: Y = 1).
// One lane = one column of 4 elements of all M workers.  Workers are loaded in chain order
// (row (b+ky) mod Y, column (a+kx) mod X for part a*Y+b), so register indices are static and only
// the addresses depend on the part.  Handles whole packed words only (n_cols is a multiple of 16,
// every column has its 4 elements); pointers and row strides need dword alignment only, the
// 128-bit accesses take any dword-aligned address.  A ragged tail goes to the generic kernel.
//
// Occupancy is throttled from the host (dynamic LDS that the kernel never touches): with 25
// concurrent streams HBM delivers most when each CU keeps only about 40-50 KB of reads in flight;
// more resident wavefronts widen the window of open DRAM rows and cost up to 10 % of bandwidth.
//
// Order inside a lane, per row of the schedule: issue the row's 2X 128-bit loads (one row ahead),
// generate the row's Philox draws while they are in flight (the draws do not depend on the data),
// then consume.  The scheduling barriers keep the compiler from sinking the loads next to their
// uses, which would leave only two loads in flight per wavefront.
// -------------------------------------------------------------------------------------------------
//
// APPLY: the model update of Algorithm 2 in the same pass, x <- x - update (x is one more read and
// one more write stream); `update` may then be NULL.  Without APPLY the kernel never looks at x.
template <int X, int Y, bool APPLY, bool GROUPED>
__global__ void __launch_bounds__(kSyncBlock)
sync_step_kernel(const float *__restrict__ g, float *__restrict__ c, float *__restrict__ update,
                 uint32_t *__restrict__ bits32, uint64_t n_cols, uint64_t ld, uint32_t scale_bits,
                 uint32_t key0, uint32_t key1, PartTable parts, float *__restrict__ x_model)
{
    constexpr int M = X * Y;
    // Consecutive workgroup ids go to consecutive XCDs, each with its own L2.  When the rows do not
    // start on 128-byte lines a tile shares its first and last line with its neighbours; GROUPED
    // gives each XCD runs of parts.xcd_group consecutive tiles, so that the second request for such
    // a line hits that L2.  (A separate instantiation: the plain one is sensitive to every
    // instruction added before its loads.)
    uint32_t tile = blockIdx.x;
    if (GROUPED) {
        const uint32_t xcd_group = parts.xcd_group;
        const uint32_t span = 8u * xcd_group;
        const uint32_t full = (gridDim.x / span) * span;
        if (tile < full) {
            const uint32_t xcd = tile % 8u, j = tile / 8u;
            tile = ((j / xcd_group) * 8u + xcd) * xcd_group + (j % xcd_group);
        }
    }
    const uint64_t col = static_cast<uint64_t>(tile) * kSyncBlock + threadIdx.x;
    const uint32_t w = static_cast<uint32_t>(col >> 4);
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    uint32_t nib = 0;

    if (col < n_cols) {
        const uint64_t e = col << 2;

        // Algorithm 1, split step: which part does this packed word belong to
        uint32_t f = 0;
#pragma unroll
        for (int k = 1; k < M; ++k)
            f += (w >= parts.bound[k]) ? 1u : 0u;
        const uint32_t a = f / Y;
        const uint32_t b = f % Y;

        // Rows are taken one after the other (a ring is a single row).  The 2X loads of a row are
        // issued one row ahead of the row being folded, and the row's Philox draws run while they
        // are in flight; the scheduling barriers keep that order.
        size_t off[Y][X];
        f32x4 s[Y][X];              // compensated gradient s = g + c, kept for the compensation update
        f32x4 gv[2][X], cv[2][X];   // the row in flight and the row being folded
        uint32_t row_res[Y][4];     // raw fp32 word whose sign is the row's merged sign, per bit
        auto fetch_row = [&](int ky) {
            uint32_t y = b + ky;
            y = (y >= Y) ? y - Y : y;
#pragma unroll
            for (int kx = 0; kx < X; ++kx) {
                uint32_t x = a + kx;
                x = (x >= X) ? x - X : x;
                off[ky][kx] = static_cast<size_t>(y * X + x) * ld + e;
                gv[ky & 1][kx] = load4_stream(g + off[ky][kx]);
                cv[ky & 1][kx] = load4_stream(c + off[ky][kx]);
            }
        };
        fetch_row(0);
        f32x4 xv = {0.0f, 0.0f, 0.0f, 0.0f};
        if (APPLY)
            xv = load4_stream(x_model + e);
        uint32_t pick_col[4] = {0, 0, 0, 0};
#pragma unroll
        for (int ky = 0; ky < Y; ++ky) {
            if (ky + 1 < Y)
                fetch_row(ky + 1);
            __builtin_amdgcn_sched_barrier(0);

            // Eq. 2 draws of this row's chain (and of the column chain's hop ky): which hop's
            // local sign is the last to be taken, for each of the lane's four bits
            uint32_t y = b + ky;
            y = (y >= Y) ? y - Y : y;
            uint32_t pick_row[4] = {0, 0, 0, 0};
#pragma unroll
            for (int h = 1; h < X; ++h) {
                uint32_t u[4];
                philox4x32_10(q, row_hop_id(y, h), w, 0u, key0, key1, u);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    pick_row[j] = (u[j] < keep_threshold(h + 1)) ? h : pick_row[j];
            }
            if (ky > 0) {
                uint32_t u[4];
                philox4x32_10(q, col_hop_id(ky), w, 0u, key0, key1, u);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    pick_col[j] = (u[j] < keep_threshold(ky + 1)) ? ky : pick_col[j];
            }
            __builtin_amdgcn_sched_barrier(0);

            // compensated gradient, then this row's chain of merges as a selection on the raw fp32 words
#pragma unroll
            for (int kx = 0; kx < X; ++kx)
                s[ky][kx] = gv[ky & 1][kx] + cv[ky & 1][kx];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t r = f32_bits(s[ky][0][j]);
#pragma unroll
                for (int h = 1; h < X; ++h)
                    r = (pick_row[j] == static_cast<uint32_t>(h)) ? f32_bits(s[ky][h][j]) : r;
                row_res[ky][j] = r;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // column chain over the row results
        uint32_t fin[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t r = row_res[0][j];
#pragma unroll
            for (int k = 1; k < Y; ++k)
                r = (pick_col[j] == static_cast<uint32_t>(k)) ? row_res[k][j] : r;
            fin[j] = r;
        }

        // global update: +scale where the final sign bit is clear, -scale where it is set
        f32x4 upd;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t sign = fin[j] & 0x80000000u;
            upd[j] = __uint_as_float(scale_bits ^ sign);
            nib |= (sign == 0u) ? (1u << j) : 0u;
        }
        if (!APPLY || update != nullptr)
            store4_stream(update + e, upd);
        if (APPLY)
            store4_stream(x_model + e, xv - upd);

        // compensation update: c <- s - update for every worker
#pragma unroll
        for (int ky = 0; ky < Y; ++ky)
#pragma unroll
            for (int kx = 0; kx < X; ++kx)
                store4_stream(c + off[ky][kx], s[ky][kx] - upd);
    }

    // final bitmap: all lanes of the wavefront take part in the cross-lane OR
    const uint32_t half = gather_half_word(nib, q);
    if (bits32 != nullptr && (q & 7u) == 0u && col < n_cols)
        bits32[2u * static_cast<size_t>(w) + (q >> 3)] = half;
}

// -------------------------------------------------------------------------------------------------
// Fused pass for any number of workers, any schedule (ring, torus, torus with a short last row,
// tree), any alignment, ragged tails.  The draws of Eq. 2 do not depend on the data and only the
// last successful draw of a chain decides a bit, so a lane evaluates the chains of its four bits
// on the draws alone and ends with the index of the one worker whose sign each bit takes
// (pick_workers_*).  Two kernels use that:
//
//   staged_step_kernel (M <= kMaxStagedWorkers): s = g + c of every worker is staged in LDS,
//     [M][64] 128-bit entries per one-wavefront workgroup.  The first batch of loads is issued
//     before the draws, which run while it is in flight; the picked workers' signs are looked up in
//     LDS and the compensation is written from LDS.  g and c are read once.
//   sweep_step_kernel (more workers than LDS can stage at a useful occupancy): "draws first,
//     gather, one sweep" -- fetch just the (at most four) picked elements of g and c, form the
//     update, then stream over the M workers once, kSweepBatch at a time.  Nothing is staged; the
//     lines the gather touched are fetched again by the sweep when they have left the L2 by then
//     (measured at M = 64: 1.25 x the algorithmic reads).
//
// Both cover columns col_begin .. ceil(d/4)-1 (col_begin is a multiple of 16).
// -------------------------------------------------------------------------------------------------
constexpr int kSweepBatch = 8;   // workers whose loads are issued back to back (sweep, full-precision round)

enum SweepSchedule { kSweepTorus = 0, kSweepRaggedTorus = 1, kSweepTree = 2 };

struct SweepShape {
    uint32_t M;           // workers
    uint32_t X, Y;        // torus: columns, rows (ring: X = M, Y = 1)
    uint32_t X_last;      // ragged torus: workers of the last row
    uint32_t top_level;   // tree: ceil(log2 M)
};

// Ring or torus whose rows are all X long: worker picked by each of the lane's four bits.
// Column chain first (which row result survives, per bit), then the chain of that row.  With up
// to four rows every row's chain is evaluated once and serves all four bits (Y*(X-1) calls);
// with more rows each bit evaluates the chain of its own row (4*(X-1) calls).
__device__ __forceinline__ void pick_workers_torus(uint32_t w, uint32_t q, uint32_t key0, uint32_t key1,
                                                   const SweepShape &shape, const PartTable &parts,
                                                   const ThresholdTable &thresholds, uint32_t worker[4])
{
    const uint32_t X = shape.X, Y = shape.Y, M = shape.M;
    uint32_t f = 0;                                   // Algorithm 1, split step
    for (uint32_t k = 1; k < M; ++k)
        f += (w >= parts.bound[k]) ? 1u : 0u;
    const uint32_t a = f / Y;
    const uint32_t b = f % Y;

    uint32_t pick_col[4] = {0, 0, 0, 0};
    for (uint32_t ky = 1; ky < Y; ++ky) {
        uint32_t u[4];
        philox4x32_10(q, col_hop_id(ky), w, 0u, key0, key1, u);
        const uint32_t thr = thresholds.thr[ky + 1];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            pick_col[j] = (u[j] < thr) ? ky : pick_col[j];
    }
    if (Y <= 4) {
        for (uint32_t ky = 0; ky < Y; ++ky) {
            uint32_t y = b + ky;
            y = (y >= Y) ? y - Y : y;
            uint32_t pick_row[4] = {0, 0, 0, 0};
            for (uint32_t kx = 1; kx < X; ++kx) {
                uint32_t u[4];
                philox4x32_10(q, row_hop_id(y, kx), w, 0u, key0, key1, u);
                const uint32_t thr = thresholds.thr[kx + 1];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    pick_row[j] = (u[j] < thr) ? kx : pick_row[j];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t x = a + pick_row[j];
                x = (x >= X) ? x - X : x;
                worker[j] = (pick_col[j] == ky) ? y * X + x : worker[j];
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t y = b + pick_col[j];
            y = (y >= Y) ? y - Y : y;
            uint32_t pick_row = 0;
            for (uint32_t kx = 1; kx < X; ++kx) {
                uint32_t u[4];
                philox4x32_10(q, row_hop_id(y, kx), w, 0u, key0, key1, u);
                pick_row = (u[j] < thresholds.thr[kx + 1]) ? kx : pick_row;
            }
            uint32_t x = a + pick_row;
            x = (x >= X) ? x - X : x;
            worker[j] = y * X + x;
        }
    }
}

// Torus whose last row is short (M is not a multiple of the X columns): rows of X workers, the
// last one of X_last; the row chains run over the row's own length from column a mod X_y, and the
// column merges are weighted by the workers each side stands for.  parts.bound[0..X] holds the X
// row-parts; the Y sub-parts of a row-part follow the same floor rule and are found arithmetically.
__device__ __forceinline__ void pick_workers_ragged(uint32_t w, uint32_t q, uint32_t key0, uint32_t key1,
                                                    const SweepShape &shape, const PartTable &parts,
                                                    const ThresholdTable &thresholds, uint32_t worker[4])
{
    const uint32_t X = shape.X, Y = shape.Y, X_last = shape.X_last;
    uint32_t a = 0;                                   // split step: row-part a, then sub-part b of it
    for (uint32_t k = 1; k < X; ++k)
        a += (w >= parts.bound[k]) ? 1u : 0u;
    const uint32_t lo = parts.bound[a];
    const uint64_t n_part = parts.bound[a + 1] - lo;
    uint32_t b = 0;
    for (uint32_t k = 1; k < Y; ++k)
        b += (w >= lo + static_cast<uint32_t>((k * n_part) / Y)) ? 1u : 0u;

    // column chain: which row result survives, per bit (weighted draws)
    uint32_t pick_col[4] = {0, 0, 0, 0};
    uint32_t gathered = (b + 1u == Y) ? X_last : X;
    for (uint32_t k = 1; k < Y; ++k) {
        uint32_t y = b + k;
        y = (y >= Y) ? y - Y : y;
        const uint32_t w_local = (y + 1u == Y) ? X_last : X;
        const uint32_t thr = weighted_threshold(gathered, w_local);
        uint32_t u[4];
        philox4x32_10(q, col_hop_id(k), w, 0u, key0, key1, u);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            pick_col[j] = (u[j] < thr) ? k : pick_col[j];
        gathered += w_local;
    }
    if (Y <= 4) {
        for (uint32_t k = 0; k < Y; ++k) {
            uint32_t y = b + k;
            y = (y >= Y) ? y - Y : y;
            const uint32_t Xy = (y + 1u == Y) ? X_last : X;
            uint32_t pick_row[4] = {0, 0, 0, 0};
            for (uint32_t h = 1; h < Xy; ++h) {
                uint32_t u[4];
                philox4x32_10(q, row_hop_id(y, h), w, 0u, key0, key1, u);
                const uint32_t thr = thresholds.thr[h + 1];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    pick_row[j] = (u[j] < thr) ? h : pick_row[j];
            }
            const uint32_t a_y = a % Xy;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t x = a_y + pick_row[j];
                x = (x >= Xy) ? x - Xy : x;
                worker[j] = (pick_col[j] == k) ? y * X + x : worker[j];
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t y = b + pick_col[j];
            y = (y >= Y) ? y - Y : y;
            const uint32_t Xy = (y + 1u == Y) ? X_last : X;
            uint32_t pick_row = 0;
            for (uint32_t h = 1; h < Xy; ++h) {
                uint32_t u[4];
                philox4x32_10(q, row_hop_id(y, h), w, 0u, key0, key1, u);
                pick_row = (u[j] < thresholds.thr[h + 1]) ? h : pick_row;
            }
            uint32_t x = a % Xy + pick_row;
            x = (x >= Xy) ? x - Xy : x;
            worker[j] = y * X + x;
        }
    }
}

// Binary reduction tree: only the merges on the way from the root to the chosen leaf decide a bit
// (all draws are independent), so every bit walks down the tree with at most ceil(log2 M) draws.
// The merge at the root is the same for the four bits and is drawn once.
__device__ __forceinline__ void pick_workers_tree(uint32_t w, uint32_t q, uint32_t key0, uint32_t key1,
                                                  const SweepShape &shape, uint32_t worker[4])
{
    const uint32_t M = shape.M;
    uint32_t level = shape.top_level;
    uint32_t k4[4] = {0, 0, 0, 0};
    if (level > 0) {
        --level;
        const uint32_t stride = 1u << level;          // stride < M by the definition of top_level
        const uint32_t w_recv = (M - stride < stride) ? (M - stride) : stride;
        const uint32_t thr = (w_recv == stride) ? 0x80000000u : weighted_threshold(w_recv, stride);
        uint32_t u[4];
        philox4x32_10(q, tree_hop_id(level, 0u), w, 0u, key0, key1, u);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            k4[j] = (u[j] < thr) ? 0u : stride;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t k = k4[j];
        for (uint32_t l = level; l-- > 0;) {
            const uint32_t stride = 1u << l;
            const uint32_t src = k + stride;
            if (src >= M)
                continue;
            const uint32_t w_recv = (M - src < stride) ? (M - src) : stride;
            const uint32_t thr = (w_recv == stride) ? 0x80000000u : weighted_threshold(w_recv, stride);
            uint32_t u[4];
            philox4x32_10(q, tree_hop_id(l, k), w, 0u, key0, key1, u);
            k = (u[j] < thr) ? k : src;
        }
        worker[j] = k;
    }
}

extern __shared__ __align__(16) unsigned char marsit_dynamic_lds[];

template <int SCHED, int BATCH>
__global__ void __launch_bounds__(kSyncBlock)
staged_step_kernel(const float *__restrict__ g, float *__restrict__ c, float *__restrict__ update,
                   uint32_t *__restrict__ bits32, uint64_t d, uint64_t ld, uint64_t col_begin,
                   uint32_t scale_bits, uint32_t key0, uint32_t key1, SweepShape shape, PartTable parts,
                   ThresholdTable thresholds, float *__restrict__ x_model)
{
    const uint32_t M = shape.M;
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = col_begin + static_cast<uint64_t>(blockIdx.x) * kSyncBlock + threadIdx.x;
    const uint32_t w = static_cast<uint32_t>(col >> 4);
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    uint32_t nib = 0;

    if (col < n_cols) {
        const uint64_t e = col << 2;
        const bool full = e + 4 <= d;
        const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
        const bool vec = full;
        // a lane only ever touches its own entries of the staging area, so no barrier is needed
        f32x4 *stage = reinterpret_cast<f32x4 *>(marsit_dynamic_lds) + threadIdx.x;

        // the first batch of loads goes out before the draws, which run while it is in flight.
        // A batch is straight-line code: past the last worker it loads and stages the last worker
        // again (same lines, same values) instead of branching.
        f32x4 gv[BATCH], cv[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const uint32_t mm = (static_cast<uint32_t>(i) < M) ? static_cast<uint32_t>(i) : M - 1u;
            const size_t off = static_cast<size_t>(mm) * ld + e;
            gv[i] = load4(g + off, vec, n_valid);
            cv[i] = load4(c + off, vec, n_valid);
        }
        f32x4 xv = {0.0f, 0.0f, 0.0f, 0.0f};
        if (x_model != nullptr)
            xv = load4(x_model + e, vec, n_valid);
        __builtin_amdgcn_sched_barrier(0);

        uint32_t worker[4] = {0, 0, 0, 0};
        if (SCHED == kSweepTorus)
            pick_workers_torus(w, q, key0, key1, shape, parts, thresholds, worker);
        else if (SCHED == kSweepRaggedTorus)
            pick_workers_ragged(w, q, key0, key1, shape, parts, thresholds, worker);
        else
            pick_workers_tree(w, q, key0, key1, shape, worker);
        __builtin_amdgcn_sched_barrier(0);

        // compensated gradient of every worker into LDS (Algorithm 1, first step)
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const uint32_t mm = (static_cast<uint32_t>(i) < M) ? static_cast<uint32_t>(i) : M - 1u;
            stage[static_cast<size_t>(mm) * kSyncBlock] = gv[i] + cv[i];
        }
#pragma unroll 1
        for (uint32_t m0 = BATCH; m0 < M; m0 += BATCH) {
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                const uint32_t mm = (m0 + i < M) ? m0 + i : M - 1u;
                const size_t off = static_cast<size_t>(mm) * ld + e;
                gv[i] = load4(g + off, vec, n_valid);
                cv[i] = load4(c + off, vec, n_valid);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                const uint32_t mm = (m0 + i < M) ? m0 + i : M - 1u;
                stage[static_cast<size_t>(mm) * kSyncBlock] = gv[i] + cv[i];
            }
        }

        // global update from the picked workers' signs
        f32x4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (static_cast<uint32_t>(j) < n_valid) {
                const f32x4 sv = stage[static_cast<size_t>(worker[j]) * kSyncBlock];
                const uint32_t sign = f32_bits(sv[j]) & 0x80000000u;
                upd[j] = __uint_as_float(scale_bits ^ sign);
                nib |= (sign == 0u) ? (1u << j) : 0u;
            }
        }
        if (update != nullptr)
            store4<MARSIT_STREAMING_STORES>(update + e, upd, vec, n_valid);
        if (x_model != nullptr)       // Algorithm 2, model update in the same pass
            store4<MARSIT_STREAMING_STORES>(x_model + e, xv - upd, vec, n_valid);

        // compensation update c <- s - update, s from LDS
#pragma unroll 4
        for (uint32_t m = 0; m < M; ++m) {
            const f32x4 sv = stage[static_cast<size_t>(m) * kSyncBlock];
            store4<MARSIT_STREAMING_STORES>(c + static_cast<size_t>(m) * ld + e, sv - upd, vec, n_valid);
        }
    }

    const uint32_t half = gather_half_word(nib, q);
    if (bits32 != nullptr && (q & 7u) == 0u && static_cast<uint64_t>(w) * 64u < d)
        bits32[2u * static_cast<size_t>(w) + (q >> 3)] = half;
}

template <int SCHED>
__global__ void __launch_bounds__(kSyncBlock)
sweep_step_kernel(const float *__restrict__ g, float *__restrict__ c, float *__restrict__ update,
                  uint32_t *__restrict__ bits32, uint64_t d, uint64_t ld, uint64_t col_begin,
                  uint32_t scale_bits, uint32_t key0, uint32_t key1, SweepShape shape, PartTable parts,
                  ThresholdTable thresholds, float *__restrict__ x_model)
{
    const uint32_t M = shape.M;
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = col_begin + static_cast<uint64_t>(blockIdx.x) * kSyncBlock + threadIdx.x;
    const uint32_t w = static_cast<uint32_t>(col >> 4);
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    uint32_t nib = 0;

    if (col < n_cols) {
        const uint64_t e = col << 2;
        const bool full = e + 4 <= d;
        const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
        const bool vec = full;

        // (1) the draws: which worker does each bit end up taking
        uint32_t worker[4] = {0, 0, 0, 0};
        if (SCHED == kSweepTorus)
            pick_workers_torus(w, q, key0, key1, shape, parts, thresholds, worker);
        else if (SCHED == kSweepRaggedTorus)
            pick_workers_ragged(w, q, key0, key1, shape, parts, thresholds, worker);
        else
            pick_workers_tree(w, q, key0, key1, shape, worker);

        // (2) gather: the picked workers' elements (ordinary loads, so the lines stay in L2 for
        // the sweep), and behind them the first batch of the sweep and the model
        float pg[4] = {0.0f, 0.0f, 0.0f, 0.0f}, pc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (static_cast<uint32_t>(j) < n_valid) {
                const size_t at = static_cast<size_t>(worker[j]) * ld + e + static_cast<uint32_t>(j);
                pg[j] = g[at];
                pc[j] = c[at];
            }
        }
        f32x4 gv[kSweepBatch], cv[kSweepBatch];
#pragma unroll
        for (int i = 0; i < kSweepBatch; ++i) {
            if (static_cast<uint32_t>(i) < M) {
                const size_t off = static_cast<size_t>(i) * ld + e;
                gv[i] = load4(g + off, vec, n_valid);
                cv[i] = load4(c + off, vec, n_valid);
            }
        }
        f32x4 xv = {0.0f, 0.0f, 0.0f, 0.0f};
        if (x_model != nullptr)
            xv = load4(x_model + e, vec, n_valid);
        __builtin_amdgcn_sched_barrier(0);

        // global update: +scale where the picked sign bit is clear, -scale where it is set
        f32x4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (static_cast<uint32_t>(j) < n_valid) {
                const uint32_t sign = f32_bits(pg[j] + pc[j]) & 0x80000000u;   // compensated gradient's sign
                upd[j] = __uint_as_float(scale_bits ^ sign);
                nib |= (sign == 0u) ? (1u << j) : 0u;
            }
        }
        if (update != nullptr)
            store4<MARSIT_STREAMING_STORES>(update + e, upd, vec, n_valid);
        if (x_model != nullptr)       // Algorithm 2, model update in the same pass
            store4<MARSIT_STREAMING_STORES>(x_model + e, xv - upd, vec, n_valid);

        // (3) the sweep: compensation update c <- (g + c) - update for every worker
#pragma unroll 1
        for (uint32_t m0 = 0; m0 < M; m0 += kSweepBatch) {
#pragma unroll
            for (int i = 0; i < kSweepBatch; ++i) {
                if (m0 + i < M) {
                    const size_t off = static_cast<size_t>(m0 + i) * ld + e;
                    store4<MARSIT_STREAMING_STORES>(c + off, (gv[i] + cv[i]) - upd, vec, n_valid);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < kSweepBatch; ++i) {
                if (m0 + kSweepBatch + i < M) {
                    const size_t off = static_cast<size_t>(m0 + kSweepBatch + i) * ld + e;
                    gv[i] = load4(g + off, vec, n_valid);
                    cv[i] = load4(c + off, vec, n_valid);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    const uint32_t half = gather_half_word(nib, q);
    if (bits32 != nullptr && (q & 7u) == 0u && static_cast<uint64_t>(w) * 64u < d)
        bits32[2u * static_cast<size_t>(w) + (q >> 3)] = half;
}

// -------------------------------------------------------------------------------------------------
// Fused pass over a binary reduction tree (whole vectors, no parts): at level l worker
// k = 0, 2*2^l, ... folds the vector of worker k + 2^l into its own; each side stands for the
// workers of its subtree.  Same lane layout and launch shape as the ring kernel.
// -------------------------------------------------------------------------------------------------
template <int M, bool APPLY>
__global__ void __launch_bounds__(kSyncBlock)
tree_step_kernel(const float *__restrict__ g, float *__restrict__ c, float *__restrict__ update,
                 uint32_t *__restrict__ bits32, uint64_t n_cols, uint64_t ld, uint32_t scale_bits,
                 uint32_t key0, uint32_t key1, float *__restrict__ x_model)
{
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kSyncBlock + threadIdx.x;
    const uint32_t w = static_cast<uint32_t>(col >> 4);
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    uint32_t nib = 0;

    if (col < n_cols) {
        const uint64_t e = col << 2;
        f32x4 gv[M], cv[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            gv[m] = load4_stream(g + static_cast<size_t>(m) * ld + e);
            cv[m] = load4_stream(c + static_cast<size_t>(m) * ld + e);
        }
        f32x4 xv = {0.0f, 0.0f, 0.0f, 0.0f};
        if (APPLY)
            xv = load4_stream(x_model + e);
        __builtin_amdgcn_sched_barrier(0);

        // Draws first, data later: every node of the tree carries, per bit, the index of the worker
        // whose sign it currently stands for; a merge keeps the receiver's or takes the sender's.
        // After the last level node 0 holds the picked worker of every bit.
        uint32_t pick[4];
        {
            uint32_t leaf[M][4];
#pragma unroll
            for (int m = 0; m < M; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    leaf[m][j] = m;
#pragma unroll
            for (int stride = 1, level = 0; stride < M; stride *= 2, ++level) {
#pragma unroll
                for (int k = 0; k + stride < M; k += 2 * stride) {
                    const int src = k + stride;
                    const uint32_t w_recv = (M - src < stride) ? (M - src) : stride;
                    uint32_t u[4];
                    philox4x32_10(q, tree_hop_id(level, k), w, 0u, key0, key1, u);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        leaf[k][j] = (u[j] < weighted_threshold(w_recv, stride)) ? leaf[k][j] : leaf[src][j];
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                pick[j] = leaf[0][j];
        }
        __builtin_amdgcn_sched_barrier(0);

        f32x4 s[M];
#pragma unroll
        for (int m = 0; m < M; ++m)
            s[m] = gv[m] + cv[m];

        // the picked worker's raw fp32 word, per bit
        uint32_t fin[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t r = f32_bits(s[0][j]);
#pragma unroll
            for (int m = 1; m < M; ++m)
                r = (pick[j] == static_cast<uint32_t>(m)) ? f32_bits(s[m][j]) : r;
            fin[j] = r;
        }

        f32x4 upd;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t sign = fin[j] & 0x80000000u;
            upd[j] = __uint_as_float(scale_bits ^ sign);
            nib |= (sign == 0u) ? (1u << j) : 0u;
        }
        if (!APPLY || update != nullptr)
            store4_stream(update + e, upd);
        if (APPLY)
            store4_stream(x_model + e, xv - upd);
#pragma unroll
        for (int m = 0; m < M; ++m)
            store4_stream(c + static_cast<size_t>(m) * ld + e, s[m] - upd);
    }

    const uint32_t half = gather_half_word(nib, q);
    if (bits32 != nullptr && (q & 7u) == 0u && col < n_cols)
        bits32[2u * static_cast<size_t>(w) + (q >> 3)] = half;
}

// -------------------------------------------------------------------------------------------------
// Full-precision round (Algorithm 1, branch mod(t,K) == 0) for M simulated workers.
// -------------------------------------------------------------------------------------------------
// Any worker count, any alignment, ragged tails: one-wavefront workgroups, the workers taken
// kSweepBatch at a time with the batch's loads issued back to back.  TWO_IN_FLIGHT (more than 24
// workers): the next batch is requested before the current one is consumed, at two wavefronts per
// CU (measured: M = 32: 73 % against 70 % of the HBM peak, M = 64: 68-69 % against 66 %; up to 24
// workers the single-batch form with three or four wavefronts is the faster one: M = 9: 79 %
// against 72 %, M = 24: 74 % against 73 %).
template <bool TWO_IN_FLIGHT>
__global__ void __launch_bounds__(kSyncBlock)
full_sync_kernel(const float *__restrict__ g, float *__restrict__ c, float *__restrict__ update,
                 uint32_t M, uint64_t d, uint64_t ld, uint64_t col_begin,
                 float *__restrict__ x_model)
{
    constexpr int B = kSweepBatch;
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = col_begin + static_cast<uint64_t>(blockIdx.x) * kSyncBlock + threadIdx.x;
    if (col >= n_cols)
        return;
    const uint64_t e = col << 2;
    const bool full = e + 4 <= d;
    const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
    const bool vec = full;

    // the mean of the fp32 compensated gradients: summed in double in worker order, divided in
    // double, rounded once to fp32
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4 xv = zero;
    if (x_model != nullptr)
        xv = load4(x_model + e, vec, n_valid);
    auto fetch = [&](f32x4 *gv, f32x4 *cv, uint32_t m0) {
#pragma unroll
        for (int i = 0; i < B; ++i) {
            if (m0 + i < M) {
                const size_t off = static_cast<size_t>(m0 + i) * ld + e;
                gv[i] = load4(g + off, vec, n_valid);
                cv[i] = load4(c + off, vec, n_valid);
            }
        }
    };
    auto consume = [&](const f32x4 *gv, const f32x4 *cv, uint32_t m0) {
#pragma unroll
        for (int i = 0; i < B; ++i) {
            if (m0 + i < M) {
                const f32x4 sv = gv[i] + cv[i];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[j] += static_cast<double>(sv[j]);
                store4<MARSIT_STREAMING_STORES>(c + static_cast<size_t>(m0 + i) * ld + e, zero, vec, n_valid);
            }
        }
    };
    f32x4 ga[B], ca[B];
    if (TWO_IN_FLIGHT) {
        f32x4 gb[B], cb[B];
        fetch(ga, ca, 0);
#pragma unroll 1
        for (uint32_t m0 = 0; m0 < M; m0 += 2 * B) {
            if (m0 + B < M)
                fetch(gb, cb, m0 + B);
            __builtin_amdgcn_sched_barrier(0);
            consume(ga, ca, m0);
            __builtin_amdgcn_sched_barrier(0);
            if (m0 + 2 * B < M)
                fetch(ga, ca, m0 + 2 * B);
            __builtin_amdgcn_sched_barrier(0);
            if (m0 + B < M)
                consume(gb, cb, m0 + B);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll 1
        for (uint32_t m0 = 0; m0 < M; m0 += B) {
            fetch(ga, ca, m0);
            __builtin_amdgcn_sched_barrier(0);
            consume(ga, ca, m0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const double dm = static_cast<double>(M);
    f32x4 mean;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        mean[j] = static_cast<float>(acc[j] / dm);
    if (update != nullptr)
        store4<MARSIT_STREAMING_STORES>(update + e, mean, vec, n_valid);
    if (x_model != nullptr)
        store4<MARSIT_STREAMING_STORES>(x_model + e, xv - mean, vec, n_valid);
}

// The same for a compile-time worker count, whole aligned columns only, launched like the fused
// one-bit kernel (one-wavefront workgroups, all 2M loads issued up front, throttled occupancy):
// the traffic pattern is the same 2M read streams and M+1 write streams.
template <int M, bool APPLY>
__global__ void __launch_bounds__(kSyncBlock)
full_sync_fast_kernel(const float *__restrict__ g, float *__restrict__ c,
                      float *__restrict__ update, uint64_t n_cols, uint64_t ld,
                      float *__restrict__ x_model)
{
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kSyncBlock + threadIdx.x;
    if (col >= n_cols)
        return;
    const uint64_t e = col << 2;
    f32x4 gv[M], cv[M];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        gv[m] = load4_stream(g + static_cast<size_t>(m) * ld + e);
        cv[m] = load4_stream(c + static_cast<size_t>(m) * ld + e);
    }
    f32x4 xv = {0.0f, 0.0f, 0.0f, 0.0f};
    if (APPLY)
        xv = load4_stream(x_model + e);
    __builtin_amdgcn_sched_barrier(0);
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int m = 0; m < M; ++m) {
        const f32x4 sv = gv[m] + cv[m];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[j] += static_cast<double>(sv[j]);
    }
    const double dm = static_cast<double>(M);
    f32x4 mean;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        mean[j] = static_cast<float>(acc[j] / dm);
    if (!APPLY || update != nullptr)
        store4_stream(update + e, mean);
    if (APPLY)
        store4_stream(x_model + e, xv - mean);
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int m = 0; m < M; ++m)
        store4_stream(c + static_cast<size_t>(m) * ld + e, zero);
}

// -------------------------------------------------------------------------------------------------
// Launch shapes
// -------------------------------------------------------------------------------------------------
// One-wavefront workgroups of a fused kernel that should share a CU.  Measured on MI355X at
// 25.6 M elements, best count per shape: rings 2: 10, 3: 6-7, 4: 5, 5: 4-5, 6: 4, 7 and up: 3;
// tori 2x2: 5, 3x2 and 2x3: 4, 4x2, 3x3, 4x4: 3 -- about 21/M, i.e. 40-50 KB of loads in flight
// per CU, never fewer than 3.  The 2x4 torus keeps only two rows of two workers in flight and
// takes one more (4: 79 % of HBM peak, 3: 73.5 %).
// Tuning hook (marsit_set_fused_waves_per_cu): 0 = the table above.
static std::atomic<uint32_t> fused_waves_override{0};

inline uint32_t fused_waves_per_cu(uint32_t X, uint32_t Y)
{
    const uint32_t forced = fused_waves_override.load(std::memory_order_relaxed);
    if (forced != 0)
        return forced;
    const uint32_t M = X * Y;
    uint32_t waves = (21u + M / 2u) / M;
    if (waves < 3u)
        waves = 3u;
    if (X == 2u && Y == 4u)
        waves = 4u;
    return waves;
}

// The any-schedule kernels.  Up to kMaxStagedWorkers workers the [M][64] staging area of 128-bit
// entries (M KB per one-wavefront workgroup) is the dynamic LDS request, never less than what
// leaves room for staged_waves_per_cu() workgroups on a CU; above (fewer than three wavefronts
// would fit on a CU, too few to hide the M - 1 draws of each) the gather-and-sweep kernel runs,
// throttled like the compiled schedules by LDS it never touches.
// Measured on MI355X at 25.6 M elements (fraction of the 8 TB/s HBM peak, best wavefront count and
// batch per worker count): M = 5: 14 wavefronts, batch 4 (70 %); 7: 10, 4 (75 %); 9, 10: 8, 4
// (74-75 %); 11-18: 5, 8 (73-75 %; short last row: 7); 24, 32: 4, 8 (73 %, 72 %); 40: 69 %; 41, 48: batch 16 (66 %,
// 68 %); ring of 64 staged: 52 %, gather-and-sweep: 63 %.  A plain streaming kernel with the same
// 2M read and M + 1 write streams (the full-precision round) reaches 80 % at M = 9, 75 % at 24,
// 73 % at 32 and 69 % at 64: the fall with M is the memory system's, not these kernels'.  Keeping
// two batches of loads in flight, which helps that streaming kernel, does nothing here (measured).
constexpr uint32_t kMaxStagedWorkers = 48;

inline uint32_t staged_batch(uint32_t M)
{
    return M <= 10 ? 4u : (M <= 40 ? 8u : 16u);
}

inline uint32_t staged_waves_per_cu(uint32_t M, int sched)
{
    if (M > 20)
        return 4;
    if (M > 10)     // the short-last-row schedule spends more draws per lane and wants more wavefronts
        return sched == kSweepRaggedTorus ? 7 : 5;
    const uint32_t waves = 72u / M;
    return waves < 8u ? 8u : (waves > 14u ? 14u : waves);
}

inline uint32_t staged_lds_bytes(uint32_t M, int sched)
{
    const uint32_t need = M * static_cast<uint32_t>(kSyncBlock) * 16u;
    const uint32_t throttle = throttle_lds_bytes(staged_waves_per_cu(M, sched));
    return need > throttle ? need : throttle;
}

constexpr uint32_t kSweepWavesPerCu = 8;   // gather-and-sweep kernel; 6 to 16 measure the same

inline ThresholdTable keep_thresholds()
{
    ThresholdTable thresholds;
    thresholds.thr[0] = 0;
    thresholds.thr[1] = 0xFFFFFFFFu;
    for (uint32_t m = 2; m <= MARSIT_MAX_WORKERS; ++m)
        thresholds.thr[m] = keep_threshold(m);
    return thresholds;
}

// Launches the any-schedule kernel over columns col_begin .. ceil(d/4) - 1.
template <int SCHED>
void launch_sweep(const float *g, float *c, float *update, uint32_t *bits32, uint64_t d, uint64_t ld,
                  uint64_t col_begin, uint32_t scale_bits, uint32_t key0, uint32_t key1,
                  const SweepShape &shape, const PartTable &parts, float *x_model, hipStream_t stream)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint32_t blocks = static_cast<uint32_t>((n_cols - col_begin + kSyncBlock - 1) / kSyncBlock);
    const ThresholdTable thresholds = keep_thresholds();
    // the tree draws only ~4 log2 M times per lane, so two wavefronts per CU still hide its draws
    // and it stays staged up to 64 workers (measured at M = 64: 67 % staged, 64 % swept)
    if (shape.M > kMaxStagedWorkers && SCHED != kSweepTree) {
        hipLaunchKernelGGL((sweep_step_kernel<SCHED>), dim3(blocks), dim3(kSyncBlock),
                           throttle_lds_bytes(kSweepWavesPerCu), stream, g, c, update, bits32, d, ld, col_begin,
                           scale_bits, key0, key1, shape, parts, thresholds, x_model);
        return;
    }
    const uint32_t lds = staged_lds_bytes(shape.M, SCHED);
    switch (staged_batch(shape.M)) {
    case 4:
        hipLaunchKernelGGL((staged_step_kernel<SCHED, 4>), dim3(blocks), dim3(kSyncBlock), lds, stream, g, c,
                           update, bits32, d, ld, col_begin, scale_bits, key0, key1, shape, parts, thresholds,
                           x_model);
        break;
    case 8:
        hipLaunchKernelGGL((staged_step_kernel<SCHED, 8>), dim3(blocks), dim3(kSyncBlock), lds, stream, g, c,
                           update, bits32, d, ld, col_begin, scale_bits, key0, key1, shape, parts, thresholds,
                           x_model);
        break;
    default:
        hipLaunchKernelGGL((staged_step_kernel<SCHED, 16>), dim3(blocks), dim3(kSyncBlock), lds, stream, g, c,
                           update, bits32, d, ld, col_begin, scale_bits, key0, key1, shape, parts, thresholds,
                           x_model);
        break;
    }
}

// The tree kernel does a little less work between issuing its loads and using them and wants one
// wavefront more (measured: M = 4: 6-7 wavefronts 79 %, 5: 78 %; M = 8: 4 wavefronts 77.7 %, 3: 75 %;
// M = 16: 3 wavefronts 75 %, 4: 73 %).
inline uint32_t tree_waves_per_cu(uint32_t M)
{
    const uint32_t waves = (28u + M / 2u) / M;
    return waves < 3u ? 3u : waves;
}

template <int X, int Y>
void launch_sync_step(const float *g, float *c, float *update, uint32_t *bits32, uint64_t n_cols,
                      uint64_t ld, uint32_t scale_bits, uint32_t key0, uint32_t key1,
                      const PartTable &parts, float *x_model, hipStream_t stream)
{
    const uint32_t lds = throttle_lds_bytes(fused_waves_per_cu(X, Y));
    const uint32_t blocks = static_cast<uint32_t>((n_cols + kSyncBlock - 1) / kSyncBlock);
    // rows on 128-byte lines: plain round-robin of tiles over the XCDs is best (M = 8: 80 % of the
    // HBM peak against 77 % with runs of 8); otherwise runs of 8 tiles per XCD up to 8 workers, of 2
    // above (M = 8, ld = d + 1: 71 % against 67 %; ld = d + 8: 72.5 % against 69.5 %; M = 16,
    // ld = d + 8: 66-67 % against 63 %)
    const bool on_lines = aligned_to(g, 128) && aligned_to(c, 128) && (ld % 32u) == 0;
    if (on_lines) {
        if (x_model == nullptr)
            hipLaunchKernelGGL((sync_step_kernel<X, Y, false, false>), dim3(blocks), dim3(kSyncBlock), lds, stream,
                               g, c, update, bits32, n_cols, ld, scale_bits, key0, key1, parts, x_model);
        else
            hipLaunchKernelGGL((sync_step_kernel<X, Y, true, false>), dim3(blocks), dim3(kSyncBlock), lds, stream,
                               g, c, update, bits32, n_cols, ld, scale_bits, key0, key1, parts, x_model);
        return;
    }
    PartTable grouped = parts;
    grouped.xcd_group = (X * Y <= 8) ? 8u : 2u;
    if (x_model == nullptr)
        hipLaunchKernelGGL((sync_step_kernel<X, Y, false, true>), dim3(blocks), dim3(kSyncBlock), lds, stream,
                           g, c, update, bits32, n_cols, ld, scale_bits, key0, key1, grouped, x_model);
    else
        hipLaunchKernelGGL((sync_step_kernel<X, Y, true, true>), dim3(blocks), dim3(kSyncBlock), lds, stream,
                           g, c, update, bits32, n_cols, ld, scale_bits, key0, key1, grouped, x_model);
}

using SyncLauncher = void (*)(const float *, float *, float *, uint32_t *, uint64_t, uint64_t,
                              uint32_t, uint32_t, uint32_t, const PartTable &, float *, hipStream_t);

// Schedules with a compiled specialisation; every other shape runs the generic kernel.
SyncLauncher find_specialisation(uint32_t X, uint32_t Y)
{
#define MARSIT_CASE(XX, YY) \
    if (X == XX && Y == YY) return &launch_sync_step<XX, YY>;
    MARSIT_CASE(1, 1) MARSIT_CASE(2, 1) MARSIT_CASE(3, 1) MARSIT_CASE(4, 1) MARSIT_CASE(5, 1)
    MARSIT_CASE(6, 1) MARSIT_CASE(7, 1) MARSIT_CASE(8, 1) MARSIT_CASE(9, 1) MARSIT_CASE(10, 1)
    MARSIT_CASE(11, 1) MARSIT_CASE(12, 1) MARSIT_CASE(13, 1) MARSIT_CASE(14, 1) MARSIT_CASE(15, 1)
    MARSIT_CASE(16, 1)
    MARSIT_CASE(2, 2) MARSIT_CASE(3, 2) MARSIT_CASE(2, 3) MARSIT_CASE(4, 2) MARSIT_CASE(2, 4)
    MARSIT_CASE(3, 3) MARSIT_CASE(4, 4)
#undef MARSIT_CASE
    return nullptr;
}

template <int M>
void launch_full_sync(const float *g, float *c, float *update, uint64_t n_cols, uint64_t ld,
                      float *x_model, hipStream_t stream)
{
    const uint32_t lds = throttle_lds_bytes(fused_waves_per_cu(M, 1));
    const uint32_t blocks = static_cast<uint32_t>((n_cols + kSyncBlock - 1) / kSyncBlock);
    if (x_model == nullptr)
        hipLaunchKernelGGL((full_sync_fast_kernel<M, false>), dim3(blocks), dim3(kSyncBlock), lds, stream,
                           g, c, update, n_cols, ld, x_model);
    else
        hipLaunchKernelGGL((full_sync_fast_kernel<M, true>), dim3(blocks), dim3(kSyncBlock), lds, stream,
                           g, c, update, n_cols, ld, x_model);
}

template <int M>
void launch_tree_step(const float *g, float *c, float *update, uint32_t *bits32, uint64_t n_cols,
                      uint64_t ld, uint32_t scale_bits, uint32_t key0, uint32_t key1, float *x_model,
                      hipStream_t stream)
{
    const uint32_t lds = throttle_lds_bytes(tree_waves_per_cu(M));
    const uint32_t blocks = static_cast<uint32_t>((n_cols + kSyncBlock - 1) / kSyncBlock);
    if (x_model == nullptr)
        hipLaunchKernelGGL((tree_step_kernel<M, false>), dim3(blocks), dim3(kSyncBlock), lds, stream, g, c,
                           update, bits32, n_cols, ld, scale_bits, key0, key1, x_model);
    else
        hipLaunchKernelGGL((tree_step_kernel<M, true>), dim3(blocks), dim3(kSyncBlock), lds, stream, g, c,
                           update, bits32, n_cols, ld, scale_bits, key0, key1, x_model);
}

using TreeLauncher = void (*)(const float *, float *, float *, uint32_t *, uint64_t, uint64_t, uint32_t,
                              uint32_t, uint32_t, float *, hipStream_t);

TreeLauncher find_tree(uint32_t M)
{
    switch (M) {
    case 1: return &launch_tree_step<1>;
    case 2: return &launch_tree_step<2>;
    case 3: return &launch_tree_step<3>;
    case 4: return &launch_tree_step<4>;
    case 5: return &launch_tree_step<5>;
    case 6: return &launch_tree_step<6>;
    case 7: return &launch_tree_step<7>;
    case 8: return &launch_tree_step<8>;
    case 12: return &launch_tree_step<12>;
    case 16: return &launch_tree_step<16>;
    default: return nullptr;
    }
}

using FullSyncLauncher = void (*)(const float *, float *, float *, uint64_t, uint64_t, float *, hipStream_t);

FullSyncLauncher find_full_sync(uint32_t M)
{
    switch (M) {
    case 1: return &launch_full_sync<1>;
    case 2: return &launch_full_sync<2>;
    case 3: return &launch_full_sync<3>;
    case 4: return &launch_full_sync<4>;
    case 5: return &launch_full_sync<5>;
    case 6: return &launch_full_sync<6>;
    case 7: return &launch_full_sync<7>;
    case 8: return &launch_full_sync<8>;
    case 12: return &launch_full_sync<12>;
    case 16: return &launch_full_sync<16>;
    default: return nullptr;
    }
}

}   // namespace marsit

using namespace marsit;

// The one-bit pass; x_model != NULL: with the model update x <- x - update in the same kernels
// (update_out may then be NULL).
static int ring_step_impl(const float *g, float *c, float *update_out, uint64_t *bits_out,
                          float *x_model, uint32_t M, uint64_t d, uint64_t ld, float scale,
                          uint64_t seed, uint32_t grid_x, void *stream)
{
    if (g == nullptr || c == nullptr || (update_out == nullptr && x_model == nullptr) || M == 0 ||
        M > MARSIT_MAX_WORKERS || ld < d || !std::isfinite(scale) || d > kMaxElements)
        return MARSIT_EINVAL;
    const uint32_t X = (grid_x == 0) ? M : grid_x;
    if (M % X != 0)
        return MARSIT_EINVAL;
    const uint32_t Y = M / X;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4) ||
        !aligned_to(bits_out, 8) || !aligned_to(x_model, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;

    const uint64_t n_words = (d + 63) / 64;
    uint64_t bounds[MARSIT_MAX_WORKERS + 1];
    split_bounds_host(n_words, M, grid_x, bounds);
    PartTable parts;
    parts.xcd_group = 1;
    for (uint32_t k = 0; k <= MARSIT_MAX_WORKERS; ++k)
        parts.bound[k] = static_cast<uint32_t>(k <= M ? bounds[k] : n_words);

    const uint32_t scale_bits = float_bits_host(scale);
    const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
    uint32_t *bits32 = reinterpret_cast<uint32_t *>(bits_out);
    hipStream_t s = static_cast<hipStream_t>(stream);

    // Whole packed words go to the kernel compiled for this schedule, the ragged last word (and
    // every input without a compiled schedule) to the generic kernel.  The two write disjoint
    // outputs.
    const SyncLauncher fast = find_specialisation(X, Y);
    uint64_t generic_col_begin = 0;
    if (fast != nullptr) {
        const uint64_t fast_cols = (d / 64) * 16;
        if (fast_cols > 0) {
            fast(g, c, update_out, bits32, fast_cols, ld, scale_bits, key0, key1, parts, x_model, s);
            const int rc = finish_launch();
            if (rc != MARSIT_OK)
                return rc;
        }
        generic_col_begin = fast_cols;
    }
    const uint64_t n_cols = (d + 3) >> 2;
    if (generic_col_begin < n_cols) {
        const SweepShape shape = {M, X, Y, X, 0u};
        launch_sweep<kSweepTorus>(g, c, update_out, bits32, d, ld, generic_col_begin, scale_bits, key0, key1,
                                  shape, parts, x_model, s);
        return finish_launch();
    }
    return MARSIT_OK;
}

// The one-bit pass over a torus of grid_x columns whose last row may be short.  A grid that divides
// M is the plain torus (or the ring) and goes to ring_step_impl.
static int ragged_torus_impl(const float *g, float *c, float *update_out, uint64_t *bits_out,
                             float *x_model, uint32_t M, uint64_t d, uint64_t ld, float scale,
                             uint64_t seed, uint32_t grid_x, void *stream)
{
    if (M == 0 || M > MARSIT_MAX_WORKERS || grid_x == 0 || grid_x > M)
        return MARSIT_EINVAL;
    if (M % grid_x == 0)
        return ring_step_impl(g, c, update_out, bits_out, x_model, M, d, ld, scale, seed, grid_x, stream);
    if (g == nullptr || c == nullptr || (update_out == nullptr && x_model == nullptr) || ld < d ||
        !std::isfinite(scale) || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4) ||
        !aligned_to(bits_out, 8) || !aligned_to(x_model, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;

    const uint32_t X = grid_x, Y = (M + X - 1) / X, X_last = M - (Y - 1) * X;
    const uint64_t n_words = (d + 63) / 64;
    uint64_t row_bounds[MARSIT_MAX_WORKERS + 1];
    split_bounds_host(n_words, X, 0, row_bounds);          // the X row-parts (a ring split in X)
    PartTable parts;
    parts.xcd_group = 1;
    for (uint32_t k = 0; k <= MARSIT_MAX_WORKERS; ++k)
        parts.bound[k] = static_cast<uint32_t>(k <= X ? row_bounds[k] : n_words);
    const uint32_t scale_bits = float_bits_host(scale);
    const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
    const SweepShape shape = {M, X, Y, X_last, 0u};
    launch_sweep<kSweepRaggedTorus>(g, c, update_out, reinterpret_cast<uint32_t *>(bits_out), d, ld, 0,
                                    scale_bits, key0, key1, shape, parts, x_model,
                                    static_cast<hipStream_t>(stream));
    return finish_launch();
}

// The full-precision round; x_model as in ring_step_impl.
static int full_sync_impl(const float *g, float *c, float *update_out, float *x_model, uint32_t M,
                          uint64_t d, uint64_t ld, void *stream)
{
    if (g == nullptr || c == nullptr || (update_out == nullptr && x_model == nullptr) || M == 0 ||
        M > MARSIT_MAX_WORKERS || ld < d || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4) || !aligned_to(x_model, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint64_t col_begin = 0;
    const FullSyncLauncher fast = find_full_sync(M);
    if (fast != nullptr && d >= 4) {
        col_begin = d / 4;
        fast(g, c, update_out, col_begin, ld, x_model, s);
        const int rc = finish_launch();
        if (rc != MARSIT_OK)
            return rc;
    }
    const uint64_t n_cols = (d + 3) >> 2;
    if (col_begin < n_cols) {
        const uint32_t blocks = static_cast<uint32_t>((n_cols - col_begin + kSyncBlock - 1) / kSyncBlock);
        if (M > 24)
            hipLaunchKernelGGL(full_sync_kernel<true>, dim3(blocks), dim3(kSyncBlock), throttle_lds_bytes(2), s, g, c,
                               update_out, M, d, ld, col_begin, x_model);
        else
            hipLaunchKernelGGL(full_sync_kernel<false>, dim3(blocks), dim3(kSyncBlock),
                               throttle_lds_bytes(M <= 16 ? 4 : 3), s, g, c, update_out, M, d, ld, col_begin, x_model);
        return finish_launch();
    }
    return MARSIT_OK;
}

extern "C" {

int marsit_set_fused_waves_per_cu(uint32_t waves)
{
    if (waves != 0 && (waves < 2 || waves > 32))
        return MARSIT_EINVAL;
    fused_waves_override.store(waves, std::memory_order_relaxed);
    return MARSIT_OK;
}

int marsit_ring_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                         uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                         uint32_t grid_x, void *stream)
{
    if (update_out == nullptr)
        return MARSIT_EINVAL;
    return ring_step_impl(g, c, update_out, bits_out, nullptr, M, d, ld, scale, seed, grid_x, stream);
}

static int tree_step_impl(const float *g, float *c, float *update_out, uint64_t *bits_out,
                          float *x_model, uint32_t M, uint64_t d, uint64_t ld, float scale,
                          uint64_t seed, void *stream)
{
    if (g == nullptr || c == nullptr || (update_out == nullptr && x_model == nullptr) || M == 0 ||
        M > MARSIT_MAX_WORKERS || ld < d || !std::isfinite(scale) || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4) ||
        !aligned_to(bits_out, 8) || !aligned_to(x_model, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const uint32_t scale_bits = float_bits_host(scale);
    const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
    uint32_t *bits32 = reinterpret_cast<uint32_t *>(bits_out);
    hipStream_t s = static_cast<hipStream_t>(stream);

    const TreeLauncher fast = find_tree(M);
    uint64_t generic_col_begin = 0;
    if (fast != nullptr) {
        const uint64_t fast_cols = (d / 64) * 16;
        if (fast_cols > 0) {
            fast(g, c, update_out, bits32, fast_cols, ld, scale_bits, key0, key1, x_model, s);
            const int rc = finish_launch();
            if (rc != MARSIT_OK)
                return rc;
        }
        generic_col_begin = fast_cols;
    }
    const uint64_t n_cols = (d + 3) >> 2;
    if (generic_col_begin < n_cols) {
        uint32_t top_level = 0;
        while ((1u << top_level) < M)
            ++top_level;
        const SweepShape shape = {M, M, 1u, M, top_level};
        PartTable no_parts;
        no_parts.xcd_group = 1;
        for (uint32_t k = 0; k <= MARSIT_MAX_WORKERS; ++k)
            no_parts.bound[k] = 0;                        // a tree folds whole vectors
        launch_sweep<kSweepTree>(g, c, update_out, bits32, d, ld, generic_col_begin, scale_bits, key0, key1,
                                 shape, no_parts, x_model, s);
        return finish_launch();
    }
    return MARSIT_OK;
}

int marsit_tree_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                         uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed, void *stream)
{
    if (update_out == nullptr)
        return MARSIT_EINVAL;
    return tree_step_impl(g, c, update_out, bits_out, nullptr, M, d, ld, scale, seed, stream);
}

int marsit_tree_step_apply(const float *g, float *c, float *x, float *update_out, uint64_t *bits_out,
                           uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed, void *stream)
{
    if (x == nullptr || x == update_out)
        return MARSIT_EINVAL;
    return tree_step_impl(g, c, update_out, bits_out, x, M, d, ld, scale, seed, stream);
}

int marsit_ragged_torus_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                                 uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                                 uint32_t grid_x, void *stream)
{
    if (update_out == nullptr)
        return MARSIT_EINVAL;
    return ragged_torus_impl(g, c, update_out, bits_out, nullptr, M, d, ld, scale, seed, grid_x, stream);
}

int marsit_ragged_torus_step_apply(const float *g, float *c, float *x, float *update_out,
                                   uint64_t *bits_out, uint32_t M, uint64_t d, uint64_t ld, float scale,
                                   uint64_t seed, uint32_t grid_x, void *stream)
{
    if (x == nullptr || x == update_out)
        return MARSIT_EINVAL;
    return ragged_torus_impl(g, c, update_out, bits_out, x, M, d, ld, scale, seed, grid_x, stream);
}

int marsit_full_sync(const float *g, float *c, float *update_out, uint32_t M, uint64_t d,
                     uint64_t ld, void *stream)
{
    if (update_out == nullptr)
        return MARSIT_EINVAL;
    return full_sync_impl(g, c, update_out, nullptr, M, d, ld, stream);
}

int marsit_step(uint64_t t, uint64_t K, const float *g, float *c, float *update_out,
                uint64_t *bits_out, uint32_t M, uint64_t d, uint64_t ld, float scale,
                uint64_t seed, uint32_t grid_x, void *stream)
{
    if (K == 0)
        return MARSIT_EINVAL;
    if (t % K != 0)
        return marsit_ring_step_sim(g, c, update_out, bits_out, M, d, ld, scale, seed, grid_x, stream);
    // the full-precision round takes the same arguments; check the ones it does not use itself
    if (!std::isfinite(scale) || (grid_x != 0 && (M == 0 || M % grid_x != 0)))
        return MARSIT_EINVAL;
    if (!aligned_to(bits_out, 8))
        return MARSIT_EALIGN;
    return marsit_full_sync(g, c, update_out, M, d, ld, stream);
}

int marsit_step_apply(uint64_t t, uint64_t K, const float *g, float *c, float *x, float *update_out,
                      uint64_t *bits_out, uint32_t M, uint64_t d, uint64_t ld, float scale,
                      uint64_t seed, uint32_t grid_x, void *stream)
{
    if (K == 0 || x == nullptr || x == update_out)
        return MARSIT_EINVAL;
    if (t % K != 0)
        return ring_step_impl(g, c, update_out, bits_out, x, M, d, ld, scale, seed, grid_x, stream);
    if (!std::isfinite(scale) || (grid_x != 0 && (M == 0 || M % grid_x != 0)))
        return MARSIT_EINVAL;
    if (!aligned_to(bits_out, 8))
        return MARSIT_EALIGN;
    return full_sync_impl(g, c, update_out, x, M, d, ld, stream);
}

// Algorithm 1 as a whole with the schedule as an argument (and Algorithm 2's model update when x
// is given): the caller holds no "t mod K" test and no choice between entry points.
int marsit_round(uint64_t t, uint64_t K, int schedule, uint32_t grid_x, const float *g, float *c,
                 float *x, float *update_out, uint64_t *bits_out, uint32_t M, uint64_t d, uint64_t ld,
                 float scale, uint64_t seed, void *stream)
{
    if (K == 0 || M == 0 || M > MARSIT_MAX_WORKERS || (x == nullptr && update_out == nullptr) ||
        (x != nullptr && x == update_out) || !std::isfinite(scale))
        return MARSIT_EINVAL;
    switch (schedule) {
    case MARSIT_SCHEDULE_RING:
        if (grid_x != 0 && grid_x != M)
            return MARSIT_EINVAL;
        grid_x = 0;
        break;
    case MARSIT_SCHEDULE_TORUS:
        if (grid_x == 0 || grid_x > M)
            return MARSIT_EINVAL;
        break;
    case MARSIT_SCHEDULE_TREE:
        if (grid_x != 0)
            return MARSIT_EINVAL;
        break;
    default:
        return MARSIT_EINVAL;
    }
    if (t % K == 0) {
        // the full-precision round is the same for every schedule; bits_out is only checked
        if (!aligned_to(bits_out, 8))
            return MARSIT_EALIGN;
        return full_sync_impl(g, c, update_out, x, M, d, ld, stream);
    }
    if (schedule == MARSIT_SCHEDULE_TREE)
        return tree_step_impl(g, c, update_out, bits_out, x, M, d, ld, scale, seed, stream);
    if (schedule == MARSIT_SCHEDULE_TORUS)
        return ragged_torus_impl(g, c, update_out, bits_out, x, M, d, ld, scale, seed, grid_x, stream);
    return ring_step_impl(g, c, update_out, bits_out, x, M, d, ld, scale, seed, 0, stream);
}

}   // extern "C"
