// HIP kernels (gfx950) and the C ABI of the Marsit one-bit synchronisation pass.
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
// draws generated in registers, no LDS, no matrix cores.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>

#include "marsit.h"
#include "marsit_device.hpp"

#ifndef MARSIT_STREAMING_STORES
#define MARSIT_STREAMING_STORES 1
#endif

namespace marsit {

constexpr int kBlock = 256;       // every kernel but the fused one
constexpr int kSyncBlock = 64;    // fused kernel: one wavefront per workgroup
constexpr uint64_t kMaxElements = static_cast<uint64_t>(1) << 37;   // word index stays below 2^31

// Bounds of the M parts of the packed words (word indices), passed by value in the kernel
// arguments so that a compile-time index becomes a scalar load.
struct PartTable {
    uint32_t bound[MARSIT_MAX_WORKERS + 1];
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
// every column has its 4 elements, every pointer is 16-byte aligned); a ragged tail goes to the
// generic kernel.
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
template <int X, int Y>
__global__ void __launch_bounds__(kSyncBlock)
sync_step_kernel(const float *__restrict__ g, float *__restrict__ c, float *__restrict__ update,
                 uint32_t *__restrict__ bits32, uint64_t n_cols, uint64_t ld, uint32_t scale_bits,
                 uint32_t key0, uint32_t key1, PartTable parts)
{
    constexpr int M = X * Y;
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kSyncBlock + threadIdx.x;
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
        store4_stream(update + e, upd);

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

// Staging area of the generic kernels: s = g + c of every worker for the wavefront's 64 columns,
// [M][64] 128-bit entries in dynamic LDS (M KB per one-wavefront workgroup).  A lane only ever
// touches its own entries, so no barrier is needed.  With it g and c are read once and c is
// written once, whatever M is.
extern __shared__ __align__(16) unsigned char marsit_dynamic_lds[];

constexpr int kSweepBatch = 8;   // workers whose loads are issued back to back

// Compensated gradient of Algorithm 1 for a run-time number of workers: s -> LDS.
__device__ __forceinline__ void stage_sums(const float *__restrict__ g, const float *c, f32x4 *stage,
                                           uint32_t M, uint64_t ld, uint64_t e, bool vec,
                                           uint32_t n_valid)
{
    for (uint32_t m0 = 0; m0 < M; m0 += kSweepBatch) {
        f32x4 gv[kSweepBatch], cv[kSweepBatch];
#pragma unroll
        for (int i = 0; i < kSweepBatch; ++i) {
            if (m0 + i < M) {
                const size_t off = static_cast<size_t>(m0 + i) * ld + e;
                gv[i] = load4(g + off, vec, n_valid);
                cv[i] = load4(c + off, vec, n_valid);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kSweepBatch; ++i)
            if (m0 + i < M)
                stage[static_cast<size_t>(m0 + i) * kSyncBlock + threadIdx.x] = gv[i] + cv[i];
    }
}

// Compensation update of Algorithm 1 for a run-time number of workers: c <- s - update, s from LDS.
__device__ __forceinline__ void compensate_from_stage(float *c, const f32x4 *stage, f32x4 upd,
                                                      uint32_t M, uint64_t ld, uint64_t e, bool vec,
                                                      uint32_t n_valid)
{
#pragma unroll 4
    for (uint32_t m = 0; m < M; ++m) {
        const f32x4 sv = stage[static_cast<size_t>(m) * kSyncBlock + threadIdx.x];
        store4<MARSIT_STREAMING_STORES>(c + static_cast<size_t>(m) * ld + e, sv - upd, vec, n_valid);
    }
}

// The same without the staging area (for M so large that the area would leave too few wavefronts
// per CU): g and c are read again.
__device__ __forceinline__ void compensate_from_memory(const float *__restrict__ g, float *c, f32x4 upd,
                                                       uint32_t M, uint64_t ld, uint64_t e, bool vec,
                                                       uint32_t n_valid)
{
    for (uint32_t m0 = 0; m0 < M; m0 += kSweepBatch) {
        f32x4 gv[kSweepBatch], cv[kSweepBatch];
#pragma unroll
        for (int i = 0; i < kSweepBatch; ++i) {
            if (m0 + i < M) {
                const size_t off = static_cast<size_t>(m0 + i) * ld + e;
                gv[i] = load4(g + off, vec, n_valid);
                cv[i] = load4(c + off, vec, n_valid);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kSweepBatch; ++i) {
            if (m0 + i < M) {
                const size_t off = static_cast<size_t>(m0 + i) * ld + e;
                store4<MARSIT_STREAMING_STORES>(c + off, (gv[i] + cv[i]) - upd, vec, n_valid);
            }
        }
    }
}

// Sign word of element j of worker `worker`: from the staging area, or straight from memory.
template <bool STAGED>
__device__ __forceinline__ uint32_t picked_sign(const f32x4 *stage, const float *__restrict__ g,
                                                const float *c, uint32_t worker, uint64_t ld,
                                                uint64_t e, int j)
{
    if (STAGED) {
        const f32x4 sv = stage[static_cast<size_t>(worker) * kSyncBlock + threadIdx.x];
        const float v = (j == 0) ? sv.x : (j == 1) ? sv.y : (j == 2) ? sv.z : sv.w;
        return f32_bits(v) & 0x80000000u;
    }
    const size_t at = static_cast<size_t>(worker) * ld + e + static_cast<uint32_t>(j);
    return f32_bits(g[at] + c[at]) & 0x80000000u;
}

// -------------------------------------------------------------------------------------------------
// Fused pass, any schedule (X, Y at run time), any alignment, ragged tails.  Covers columns
// col_begin .. ceil(d/4)-1 (col_begin is a multiple of 16).  s of every worker is staged in LDS,
// the chains are evaluated on the draws alone (which worker does each bit end up taking), that
// worker's sign is looked up in LDS, and the compensation is written from LDS: 12*M + 4 bytes per
// element, like the compiled schedules.
// -------------------------------------------------------------------------------------------------
template <bool STAGED>
__global__ void __launch_bounds__(kSyncBlock)
sync_step_generic_kernel(const float *__restrict__ g, float *__restrict__ c,
                         float *__restrict__ update, uint32_t *__restrict__ bits32, uint64_t d,
                         uint64_t ld, uint64_t col_begin, uint32_t scale_bits, uint32_t key0,
                         uint32_t key1, uint32_t X, uint32_t Y, bool aligned, PartTable parts,
                         ThresholdTable thresholds)
{
    const uint32_t M = X * Y;
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = col_begin + static_cast<uint64_t>(blockIdx.x) * kSyncBlock + threadIdx.x;
    const uint32_t w = static_cast<uint32_t>(col >> 4);
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    uint32_t nib = 0;

    if (col < n_cols) {
        const uint64_t e = col << 2;
        const bool full = e + 4 <= d;
        const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
        const bool vec = full && aligned;

        uint32_t f = 0;
        for (uint32_t k = 1; k < M; ++k)
            f += (w >= parts.bound[k]) ? 1u : 0u;
        const uint32_t a = f / Y;
        const uint32_t b = f % Y;

        // compensated gradient of every worker into LDS
        f32x4 *stage = reinterpret_cast<f32x4 *>(marsit_dynamic_lds);
        if (STAGED)
            stage_sums(g, c, stage, M, ld, e, vec, n_valid);

        // The draws do not depend on the data, and only the last successful draw of a chain
        // matters: find the picked worker of every bit, then look its sign up.
        // Column chain (shared by the lane's four bits): which row result survives.
        uint32_t pick_col[4] = {0, 0, 0, 0};
        for (uint32_t ky = 1; ky < Y; ++ky) {
            uint32_t u[4];
            philox4x32_10(q, col_hop_id(ky), w, 0u, key0, key1, u);
            const uint32_t thr = thresholds.thr[ky + 1];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                pick_col[j] = (u[j] < thr) ? ky : pick_col[j];
        }
        // Row chain of the surviving row.  On a ring all four bits share the one row and one call
        // per hop serves them; on a torus the rows differ per bit.
        uint32_t row_of[4], pick_row[4] = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t y = b + pick_col[j];
            row_of[j] = (y >= Y) ? y - Y : y;
        }
        if (Y == 1) {
            for (uint32_t kx = 1; kx < X; ++kx) {
                uint32_t u[4];
                philox4x32_10(q, row_hop_id(0, kx), w, 0u, key0, key1, u);
                const uint32_t thr = thresholds.thr[kx + 1];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    pick_row[j] = (u[j] < thr) ? kx : pick_row[j];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                for (uint32_t kx = 1; kx < X; ++kx) {
                    uint32_t u[4];
                    philox4x32_10(q, row_hop_id(row_of[j], kx), w, 0u, key0, key1, u);
                    pick_row[j] = (u[j] < thresholds.thr[kx + 1]) ? kx : pick_row[j];
                }
            }
        }

        f32x4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (static_cast<uint32_t>(j) < n_valid) {
                uint32_t x = a + pick_row[j];
                x = (x >= X) ? x - X : x;
                const uint32_t sign = picked_sign<STAGED>(stage, g, c, row_of[j] * X + x, ld, e, j);
                upd[j] = __uint_as_float(scale_bits ^ sign);          // global update
                nib |= (sign == 0u) ? (1u << j) : 0u;
            }
        }
        store4<MARSIT_STREAMING_STORES>(update + e, upd, vec, n_valid);

        if (STAGED)
            compensate_from_stage(c, stage, upd, M, ld, e, vec, n_valid);
        else
            compensate_from_memory(g, c, upd, M, ld, e, vec, n_valid);
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
template <int M>
__global__ void __launch_bounds__(kSyncBlock)
tree_step_kernel(const float *__restrict__ g, float *__restrict__ c, float *__restrict__ update,
                 uint32_t *__restrict__ bits32, uint64_t n_cols, uint64_t ld, uint32_t scale_bits,
                 uint32_t key0, uint32_t key1)
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
        __builtin_amdgcn_sched_barrier(0);

        // one draw per merge and bit: bit (4*i + j) of `take` = merge i keeps the receiver's own sign
        uint64_t take = 0;
        {
            int i = 0;
#pragma unroll
            for (int stride = 1, level = 0; stride < M; stride *= 2, ++level) {
#pragma unroll
                for (int k = 0; k + stride < M; k += 2 * stride, ++i) {
                    const int src = k + stride;
                    const uint32_t w_recv = (M - src < stride) ? (M - src) : stride;
                    uint32_t u[4];
                    philox4x32_10(q, tree_hop_id(level, k), w, 0u, key0, key1, u);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        take |= (u[j] < weighted_threshold(w_recv, stride))
                                    ? (static_cast<uint64_t>(1) << (4 * i + j)) : 0ull;
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        f32x4 s[M];
#pragma unroll
        for (int m = 0; m < M; ++m)
            s[m] = gv[m] + cv[m];

        // the tree, bottom level first, as selections on the raw fp32 words
        uint32_t fin[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t val[M];
#pragma unroll
            for (int m = 0; m < M; ++m)
                val[m] = f32_bits(s[m][j]);
            int i = 0;
#pragma unroll
            for (int stride = 1; stride < M; stride *= 2) {
#pragma unroll
                for (int k = 0; k + stride < M; k += 2 * stride, ++i)
                    val[k] = ((take >> (4 * i + j)) & 1ull) ? val[k] : val[k + stride];
            }
            fin[j] = val[0];
        }

        f32x4 upd;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t sign = fin[j] & 0x80000000u;
            upd[j] = __uint_as_float(scale_bits ^ sign);
            nib |= (sign == 0u) ? (1u << j) : 0u;
        }
        store4_stream(update + e, upd);
#pragma unroll
        for (int m = 0; m < M; ++m)
            store4_stream(c + static_cast<size_t>(m) * ld + e, s[m] - upd);
    }

    const uint32_t half = gather_half_word(nib, q);
    if (bits32 != nullptr && (q & 7u) == 0u && col < n_cols)
        bits32[2u * static_cast<size_t>(w) + (q >> 3)] = half;
}

// Any M, any alignment, ragged tails.  Only the merges on the way from the root to the chosen
// leaf decide a bit (all draws are independent), so every bit walks down the tree with at most
// ceil(log2 M) draws and looks up the sign of the one worker it ends at; s of every worker is
// staged in LDS as in the generic ring kernel.
template <bool STAGED>
__global__ void __launch_bounds__(kSyncBlock)
tree_step_generic_kernel(const float *__restrict__ g, float *__restrict__ c,
                         float *__restrict__ update, uint32_t *__restrict__ bits32, uint64_t d,
                         uint64_t ld, uint64_t col_begin, uint32_t scale_bits, uint32_t key0,
                         uint32_t key1, uint32_t M, uint32_t top_level, bool aligned)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = col_begin + static_cast<uint64_t>(blockIdx.x) * kSyncBlock + threadIdx.x;
    const uint32_t w = static_cast<uint32_t>(col >> 4);
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    uint32_t nib = 0;

    if (col < n_cols) {
        const uint64_t e = col << 2;
        const bool full = e + 4 <= d;
        const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
        const bool vec = full && aligned;

        f32x4 *stage = reinterpret_cast<f32x4 *>(marsit_dynamic_lds);
        if (STAGED)
            stage_sums(g, c, stage, M, ld, e, vec, n_valid);

        f32x4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
        for (uint32_t j = 0; j < n_valid; ++j) {
            uint32_t k = 0;
            for (uint32_t level = top_level; level-- > 0;) {
                const uint32_t stride = 1u << level;
                const uint32_t src = k + stride;
                if (src >= M)
                    continue;
                const uint32_t w_recv = (M - src < stride) ? (M - src) : stride;
                const uint32_t thr = (w_recv == stride) ? 0x80000000u : weighted_threshold(w_recv, stride);
                uint32_t u[4];
                philox4x32_10(q, tree_hop_id(level, k), w, 0u, key0, key1, u);
                const uint32_t uj = (j == 0) ? u[0] : (j == 1) ? u[1] : (j == 2) ? u[2] : u[3];
                k = (uj < thr) ? k : src;
            }
            const uint32_t sign = picked_sign<STAGED>(stage, g, c, k, ld, e, static_cast<int>(j));
            const float uval = __uint_as_float(scale_bits ^ sign);
            if (j == 0) upd.x = uval; else if (j == 1) upd.y = uval; else if (j == 2) upd.z = uval; else upd.w = uval;
            nib |= (sign == 0u) ? (1u << j) : 0u;
        }
        store4<MARSIT_STREAMING_STORES>(update + e, upd, vec, n_valid);
        if (STAGED)
            compensate_from_stage(c, stage, upd, M, ld, e, vec, n_valid);
        else
            compensate_from_memory(g, c, upd, M, ld, e, vec, n_valid);
    }

    const uint32_t half = gather_half_word(nib, q);
    if (bits32 != nullptr && (q & 7u) == 0u && static_cast<uint64_t>(w) * 64u < d)
        bits32[2u * static_cast<size_t>(w) + (q >> 3)] = half;
}

// -------------------------------------------------------------------------------------------------
// marsit_compress: a wavefront takes 64 consecutive elements per packed word, one per lane, and
// the 64-lane ballot of "sign bit clear" IS the word.  Four words per wavefront per trip keep
// eight independent 256-byte loads in flight.
// -------------------------------------------------------------------------------------------------
constexpr int kWordsPerWave = 4;

__global__ void __launch_bounds__(kBlock)
compress_kernel(const float *__restrict__ g, const float *__restrict__ c,
                uint64_t *__restrict__ bits, uint64_t d, uint64_t n_words)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t wave = (static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x) >> 6;
    const uint64_t w0 = wave * kWordsPerWave;
    if (w0 >= n_words)
        return;   // uniform over the wavefront

    float s[kWordsPerWave];
    bool valid[kWordsPerWave];
#pragma unroll
    for (int i = 0; i < kWordsPerWave; ++i) {
        const uint64_t e = (w0 + i) * 64u + lane;
        valid[i] = e < d;
        const float gv = valid[i] ? __builtin_nontemporal_load(g + e) : 0.0f;
        const float cv = (valid[i] && c != nullptr) ? __builtin_nontemporal_load(c + e) : 0.0f;
        s[i] = gv + cv;
    }
#pragma unroll
    for (int i = 0; i < kWordsPerWave; ++i) {
        const uint64_t word = __ballot(valid[i] && (f32_bits(s[i]) >> 31) == 0u);
        if (lane == 0 && w0 + i < n_words)
            bits[w0 + i] = word;
    }
}

// -------------------------------------------------------------------------------------------------
// marsit_hop_merge: lane = (packed word i, nibble q); one Philox call per lane.
// -------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlock)
hop_merge_kernel(const uint32_t *recv32, const uint32_t *local32, uint32_t *out32,
                 uint64_t word_begin, uint64_t n_words, uint32_t threshold, bool always_local,
                 uint32_t hop_id, uint32_t key0, uint32_t key1, const uint64_t *seed_ptr)
{
    if (seed_ptr != nullptr) {
        // seed kept in device memory: lets a captured graph be replayed with a new seed
        const uint64_t seed = *seed_ptr;
        key0 = static_cast<uint32_t>(seed);
        key1 = static_cast<uint32_t>(seed >> 32);
    }
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    const uint64_t i = col >> 4;
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    const size_t half_index = 2u * static_cast<size_t>(i) + (q >> 3);
    const uint32_t shift = (q & 7u) * 4u;
    uint32_t nib = 0;

    if (i < n_words) {
        const uint32_t r = (recv32[half_index] >> shift) & 0xFu;
        const uint32_t l = (local32[half_index] >> shift) & 0xFu;
        const uint64_t w = word_begin + i;
        uint32_t u[4];
        philox4x32_10(q, hop_id, static_cast<uint32_t>(w), static_cast<uint32_t>(w >> 32), key0,
                      key1, u);
        uint32_t t = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            t |= (always_local || u[j] < threshold) ? (1u << j) : 0u;
        nib = r ^ ((r ^ l) & t);   // t ? l : r
    }

    const uint32_t half = half_row_or(nib << shift);
    if (i < n_words && (q & 7u) == 0u)
        out32[half_index] = half;
}

// -------------------------------------------------------------------------------------------------
// marsit_decode_compensate: lane = one column of 4 elements.
// -------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlock)
decode_compensate_kernel(const uint32_t *__restrict__ bits32, const float *__restrict__ g,
                         const float *c, float *__restrict__ update, float *c_out, uint64_t d,
                         uint32_t scale_bits, bool aligned)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (col >= n_cols)
        return;
    const uint64_t e = col << 2;
    const bool full = e + 4 <= d;
    const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
    const bool vec = full && aligned;

    const uint32_t nib = (bits32[col >> 3] >> ((static_cast<uint32_t>(col) & 7u) * 4u)) & 0xFu;
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    const f32x4 sv = load4(g + e, vec, n_valid) + ((c != nullptr) ? load4(c + e, vec, n_valid) : zero);
    f32x4 upd;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        upd[j] = __uint_as_float(scale_bits ^ (((nib >> j) & 1u) ? 0u : 0x80000000u));
    if (update != nullptr)
        store4<MARSIT_STREAMING_STORES>(update + e, upd, vec, n_valid);
    store4<MARSIT_STREAMING_STORES>(c_out + e, sv - upd, vec, n_valid);
}

// -------------------------------------------------------------------------------------------------
// Full-precision round (Algorithm 1, branch mod(t,K) == 0) and the model update of Algorithm 2.
// -------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlock)
full_sync_kernel(const float *__restrict__ g, float *__restrict__ c, float *__restrict__ update,
                 uint32_t M, uint64_t d, uint64_t ld, uint64_t col_begin, bool aligned)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = col_begin + static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (col >= n_cols)
        return;
    const uint64_t e = col << 2;
    const bool full = e + 4 <= d;
    const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
    const bool vec = full && aligned;

    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 4
    for (uint32_t m = 0; m < M; ++m) {
        const size_t off = static_cast<size_t>(m) * ld + e;
        const f32x4 sv = load4(g + off, vec, n_valid) + load4(c + off, vec, n_valid);
        acc = (m == 0) ? sv : acc + sv;
        store4<MARSIT_STREAMING_STORES>(c + off, zero, vec, n_valid);
    }
    const float fm = static_cast<float>(M);
    f32x4 mean;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        mean[j] = acc[j] / fm;
    store4<MARSIT_STREAMING_STORES>(update + e, mean, vec, n_valid);
}

// The same for a compile-time worker count, whole aligned columns only, launched like the fused
// one-bit kernel (one-wavefront workgroups, all 2M loads issued up front, throttled occupancy):
// the traffic pattern is the same 2M read streams and M+1 write streams.
template <int M>
__global__ void __launch_bounds__(kSyncBlock)
full_sync_fast_kernel(const float *__restrict__ g, float *__restrict__ c,
                      float *__restrict__ update, uint64_t n_cols, uint64_t ld)
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
    __builtin_amdgcn_sched_barrier(0);
    f32x4 acc = gv[0] + cv[0];
#pragma unroll
    for (int m = 1; m < M; ++m)
        acc = acc + (gv[m] + cv[m]);
    const float fm = static_cast<float>(M);
    f32x4 mean;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        mean[j] = acc[j] / fm;
    store4_stream(update + e, mean);
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int m = 0; m < M; ++m)
        store4_stream(c + static_cast<size_t>(m) * ld + e, zero);
}

__global__ void __launch_bounds__(kBlock)
apply_update_kernel(float *__restrict__ x, const float *__restrict__ update, uint64_t d, bool aligned)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (col >= n_cols)
        return;
    const uint64_t e = col << 2;
    const bool full = e + 4 <= d;
    const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
    const bool vec = full && aligned;
    const f32x4 xv = load4<false>(x + e, vec, n_valid);
    const f32x4 uv = load4<true>(update + e, vec, n_valid);
    store4<false>(x + e, xv - uv, vec, n_valid);
}

// -------------------------------------------------------------------------------------------------
// Diagnostics of Section 3.2.2 / Fig. 2(b): sign of the non-compressed aggregate, majority vote,
// and the number of positions at which two sign bitmaps agree (numerator of the matching rate).
// -------------------------------------------------------------------------------------------------
enum VoteMode { kAggregateSign = 0, kMajorityVote = 1 };

template <int MODE>
__global__ void __launch_bounds__(kBlock)
vote_kernel(const float *__restrict__ g, const float *__restrict__ c, uint32_t *__restrict__ bits32,
            uint32_t M, uint64_t d, uint64_t ld, bool aligned)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    const uint32_t w = static_cast<uint32_t>(col >> 4);
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    uint32_t nib = 0;
    if (col < n_cols) {
        const uint64_t e = col << 2;
        const bool full = e + 4 <= d;
        const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
        const bool vec = full && aligned;
        double acc[4] = {0.0, 0.0, 0.0, 0.0};   // aggregate in double, in worker order
        uint32_t plus[4] = {0, 0, 0, 0};        // workers with a + sign
#pragma unroll 4
        for (uint32_t m = 0; m < M; ++m) {
            const size_t off = static_cast<size_t>(m) * ld + e;
            const f32x4 sv = load4(g + off, vec, n_valid) + load4(c + off, vec, n_valid);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (MODE == kAggregateSign)
                    acc[j] += static_cast<double>(sv[j]);
                else
                    plus[j] += (f32_bits(sv[j]) >> 31) ^ 1u;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool positive = (MODE == kAggregateSign)
                ? ((__double_as_longlong(acc[j]) >> 63) == 0)
                : (2u * plus[j] >= M);
            nib |= (static_cast<uint32_t>(j) < n_valid && positive) ? (1u << j) : 0u;
        }
    }
    const uint32_t half = gather_half_word(nib, q);
    if ((q & 7u) == 0u && static_cast<uint64_t>(w) * 64u < d)
        bits32[2u * static_cast<size_t>(w) + (q >> 3)] = half;
}

__global__ void zero_counter_kernel(unsigned long long *count) { *count = 0ull; }

__global__ void __launch_bounds__(kBlock)
count_matching_kernel(const uint64_t *__restrict__ a, const uint64_t *__restrict__ b, uint64_t d,
                      uint64_t n_words, unsigned long long *count)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    unsigned long long n = 0;
    if (i < n_words) {
        uint64_t same = ~(a[i] ^ b[i]);
        const uint64_t valid = d - i * 64u;                 // elements of this word that exist
        if (valid < 64u)
            same &= (static_cast<uint64_t>(1) << valid) - 1u;
        n = static_cast<unsigned long long>(__popcll(same));
    }
    // sum over the wavefront, one atomic per wavefront (integer: the order does not matter)
#pragma unroll
    for (int offset = 32; offset > 0; offset >>= 1)
        n += __shfl_down(n, offset, 64);
    if ((threadIdx.x & 63u) == 0u && n != 0ull)
        atomicAdd(count, n);
}

// -------------------------------------------------------------------------------------------------
// The strawman of Section 3.2 (a comparison point, not part of Marsit): SSDM's stochastic sign and
// one hop of cascading compression on a run of elements.
//   t[e]   = (recv ? +-recv_norm by the received sign bit : 0) + (g[e] + c[e])       (fp32)
//   norm   = sqrtf((float) sum_e (double)t[e]^2)
//   bit[e] = (double)u < (double)(0.5f + t[e] / (2.0f * norm)) * 2^32               (Appendix A)
// Three launches per hop: partial sums of squares (double, one per workgroup), the final sum in a
// fixed order, the stochastic signs.
// -------------------------------------------------------------------------------------------------
constexpr int kCascadeMaxPartials = 1024;

__device__ __forceinline__ f32x4 cascade_value(const uint32_t *recv32, const float *recv_norm,
                                               const float *g, const float *c, uint64_t col,
                                               bool vec, uint32_t n_valid)
{
    const uint64_t e = col << 2;
    f32x4 t = load4(g + e, vec, n_valid) + load4(c + e, vec, n_valid);     // compensated gradient
    if (recv32 != nullptr) {
        const float norm = *recv_norm;
        const uint32_t nib = (recv32[col >> 3] >> ((static_cast<uint32_t>(col) & 7u) * 4u)) & 0xFu;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            t[j] = (((nib >> j) & 1u) ? norm : -norm) + t[j];               // recover + aggregate
    }
    return t;
}

__global__ void __launch_bounds__(kBlock)
cascade_norm_partial_kernel(const uint32_t *recv32, const float *recv_norm, const float *g,
                            const float *c, uint64_t n, bool aligned, double *partial)
{
    __shared__ double wave_sum[kBlock / 64];
    const uint64_t n_cols = (n + 3) >> 2;
    double acc = 0.0;
    for (uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x; col < n_cols;
         col += static_cast<uint64_t>(gridDim.x) * kBlock) {
        const uint64_t e = col << 2;
        const bool full = e + 4 <= n;
        const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(n - e);
        const f32x4 t = cascade_value(recv32, recv_norm, g, c, col, full && aligned, n_valid);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (static_cast<uint32_t>(j) < n_valid)
                acc += static_cast<double>(t[j]) * static_cast<double>(t[j]);
    }
#pragma unroll
    for (int offset = 32; offset > 0; offset >>= 1)
        acc += __shfl_down(acc, offset, 64);
    if ((threadIdx.x & 63u) == 0u)
        wave_sum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
        for (int i = 0; i < kBlock / 64; ++i)
            total += wave_sum[i];
        partial[blockIdx.x] = total;
    }
}

__global__ void cascade_norm_final_kernel(const double *partial, uint32_t n_partials, float *norm_out,
                                          float *norm_copy)
{
    double total = 0.0;
    for (uint32_t i = 0; i < n_partials; ++i)
        total += partial[i];
    const float norm = sqrtf(static_cast<float>(total));
    *norm_out = norm;
    if (norm_copy != nullptr)
        *norm_copy = norm;
}

__global__ void __launch_bounds__(kBlock)
cascade_sign_kernel(const uint32_t *recv32, const float *recv_norm, const float *g, const float *c,
                    const float *norm_ptr, uint32_t *out32, uint64_t n, uint64_t word_begin,
                    uint32_t hop_id, uint32_t key0, uint32_t key1, bool aligned)
{
    const uint64_t n_cols = (n + 3) >> 2;
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    const uint64_t wl = col >> 4;                        // packed word inside this run
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    uint32_t nib = 0;
    if (col < n_cols) {
        const uint64_t e = col << 2;
        const bool full = e + 4 <= n;
        const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(n - e);
        const f32x4 t = cascade_value(recv32, recv_norm, g, c, col, full && aligned, n_valid);
        const float norm = *norm_ptr;
        const uint64_t w = word_begin + wl;
        uint32_t u[4];
        philox4x32_10(q, hop_id, static_cast<uint32_t>(w), static_cast<uint32_t>(w >> 32), key0, key1, u);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float p = 0.5f;
            if (norm != 0.0f)
                p = 0.5f + t[j] / (2.0f * norm);
            const bool plus = static_cast<double>(u[j]) < static_cast<double>(p) * 4294967296.0;
            nib |= (static_cast<uint32_t>(j) < n_valid && plus) ? (1u << j) : 0u;
        }
    }
    const uint32_t half = gather_half_word(nib, q);
    if ((q & 7u) == 0u && wl * 64u < n)
        out32[2u * static_cast<size_t>(wl) + (q >> 3)] = half;
}

__global__ void __launch_bounds__(kBlock)
cascade_decode_kernel(const uint32_t *bits32, const float *norm_ptr, float *update, uint64_t n,
                      float workers)
{
    const uint64_t e = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (e >= n)
        return;
    const float norm = *norm_ptr;
    const uint32_t bit = (bits32[e >> 5] >> (static_cast<uint32_t>(e) & 31u)) & 1u;
    update[e] = (bit ? norm : -norm) / workers;
}

// -------------------------------------------------------------------------------------------------
// Host side
// -------------------------------------------------------------------------------------------------
thread_local int tls_last_hip_error = 0;

inline int finish_launch()
{
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        tls_last_hip_error = static_cast<int>(err);
        return MARSIT_EHIP;
    }
    return MARSIT_OK;
}

inline bool aligned_to(const void *p, uintptr_t n) { return (reinterpret_cast<uintptr_t>(p) % n) == 0; }

inline uint32_t blocks_for(uint64_t n_threads)
{
    return static_cast<uint32_t>((n_threads + kBlock - 1) / kBlock);
}

inline uint32_t float_bits_host(float x)
{
    uint32_t u;
    std::memcpy(&u, &x, sizeof u);
    return u;
}

// Fine part bounds of the schedule (see marsit_split_bounds in marsit.h).
int split_bounds_host(uint64_t n_words, uint32_t M, uint32_t grid_x, uint64_t *bounds)
{
    if (bounds == nullptr || M == 0 || M > MARSIT_MAX_WORKERS)
        return MARSIT_EINVAL;
    const uint32_t X = (grid_x == 0) ? M : grid_x;
    if (X == 0 || M % X != 0)
        return MARSIT_EINVAL;
    const uint32_t Y = M / X;
    for (uint32_t a = 0; a < X; ++a) {
        const uint64_t lo = static_cast<uint64_t>((static_cast<unsigned __int128>(a) * n_words) / X);
        const uint64_t hi = static_cast<uint64_t>((static_cast<unsigned __int128>(a + 1) * n_words) / X);
        const uint64_t n = hi - lo;
        for (uint32_t b = 0; b < Y; ++b)
            bounds[a * Y + b] = lo + static_cast<uint64_t>((static_cast<unsigned __int128>(b) * n) / Y);
    }
    bounds[M] = n_words;
    return MARSIT_OK;
}

// Dynamic LDS bytes per workgroup that leave room for exactly `waves` one-wavefront workgroups of
// the fused kernel on a CU.  Measured on MI355X (25.6 M elements): the best count is 3 for M = 8
// and 16, 5 for M = 4, 10 for M = 2 -- about 40 KB of loads in flight per CU, never fewer than 3.
inline uint32_t throttle_lds_bytes(uint32_t M)
{
    constexpr uint32_t lds_per_cu = 160u * 1024u;   // gfx950; the runtime attribute reports 64 KB
    uint32_t waves = (20u + M / 2u) / M;
    if (waves < 3u)
        waves = 3u;
    // a few per cent below an even share: with an exact share one workgroup fewer fits.  At least
    // 3 workgroups per CU keeps the request under the 64 KB a launch may ask for without opting in.
    return ((lds_per_cu / waves) * 31u / 32u) & ~511u;
}

// Dynamic LDS of the generic kernels: the [M][64] staging area of 128-bit entries (M KB per
// wavefront).  Above 40 workers it would leave fewer than four wavefronts per CU, and reading g
// and c twice is faster (measured at M = 64: 62 % against 54 % of HBM peak).
constexpr uint32_t kMaxStagedWorkers = 40;
inline uint32_t generic_lds_bytes(uint32_t M)
{
    // never less than 20 KB: at most 8 wavefronts per CU (measured best for M = 9, 10: 72 % of peak
    // against 65 % with 17 wavefronts)
    const uint32_t need = M * static_cast<uint32_t>(kSyncBlock) * 16u;
    return need > 20u * 1024u ? need : 20u * 1024u;
}

template <int X, int Y>
void launch_sync_step(const float *g, float *c, float *update, uint32_t *bits32, uint64_t n_cols,
                      uint64_t ld, uint32_t scale_bits, uint32_t key0, uint32_t key1,
                      const PartTable &parts, hipStream_t stream)
{
    const uint32_t lds = throttle_lds_bytes(X * Y);
    const uint32_t blocks = static_cast<uint32_t>((n_cols + kSyncBlock - 1) / kSyncBlock);
    hipLaunchKernelGGL((sync_step_kernel<X, Y>), dim3(blocks), dim3(kSyncBlock), lds, stream, g, c,
                       update, bits32, n_cols, ld, scale_bits, key0, key1, parts);
}

using SyncLauncher = void (*)(const float *, float *, float *, uint32_t *, uint64_t, uint64_t,
                              uint32_t, uint32_t, uint32_t, const PartTable &, hipStream_t);

// Schedules with a compiled specialisation; every other shape runs the generic kernel.
SyncLauncher find_specialisation(uint32_t X, uint32_t Y)
{
#define MARSIT_CASE(XX, YY) \
    if (X == XX && Y == YY) return &launch_sync_step<XX, YY>;
    MARSIT_CASE(1, 1) MARSIT_CASE(2, 1) MARSIT_CASE(3, 1) MARSIT_CASE(4, 1) MARSIT_CASE(5, 1)
    MARSIT_CASE(6, 1) MARSIT_CASE(7, 1) MARSIT_CASE(8, 1) MARSIT_CASE(12, 1) MARSIT_CASE(16, 1)
    MARSIT_CASE(2, 2) MARSIT_CASE(3, 2) MARSIT_CASE(2, 3) MARSIT_CASE(4, 2) MARSIT_CASE(2, 4)
    MARSIT_CASE(3, 3) MARSIT_CASE(4, 4)
#undef MARSIT_CASE
    return nullptr;
}

template <int M>
void launch_full_sync(const float *g, float *c, float *update, uint64_t n_cols, uint64_t ld,
                      hipStream_t stream)
{
    const uint32_t lds = throttle_lds_bytes(M);
    const uint32_t blocks = static_cast<uint32_t>((n_cols + kSyncBlock - 1) / kSyncBlock);
    hipLaunchKernelGGL((full_sync_fast_kernel<M>), dim3(blocks), dim3(kSyncBlock), lds, stream, g, c,
                       update, n_cols, ld);
}

template <int M>
void launch_tree_step(const float *g, float *c, float *update, uint32_t *bits32, uint64_t n_cols,
                      uint64_t ld, uint32_t scale_bits, uint32_t key0, uint32_t key1,
                      hipStream_t stream)
{
    const uint32_t lds = throttle_lds_bytes(M);
    const uint32_t blocks = static_cast<uint32_t>((n_cols + kSyncBlock - 1) / kSyncBlock);
    hipLaunchKernelGGL((tree_step_kernel<M>), dim3(blocks), dim3(kSyncBlock), lds, stream, g, c, update,
                       bits32, n_cols, ld, scale_bits, key0, key1);
}

using TreeLauncher = void (*)(const float *, float *, float *, uint32_t *, uint64_t, uint64_t, uint32_t,
                              uint32_t, uint32_t, hipStream_t);

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

using FullSyncLauncher = void (*)(const float *, float *, float *, uint64_t, uint64_t, hipStream_t);

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

extern "C" {

int marsit_version(void) { return 100; }

int marsit_last_hip_error(void) { return tls_last_hip_error; }

const char *marsit_status_string(int status)
{
    switch (status) {
    case MARSIT_OK: return "ok";
    case MARSIT_EINVAL: return "invalid argument";
    case MARSIT_EALIGN: return "pointer not aligned to its element size";
    case MARSIT_EHIP: return "HIP call failed (see marsit_last_hip_error)";
    default: return "unknown status";
    }
}

void marsit_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1], out);
}

int marsit_split_bounds(uint64_t n_words, uint32_t M, uint32_t grid_x, uint64_t *bounds_out)
{
    return split_bounds_host(n_words, M, grid_x, bounds_out);
}

int marsit_compress(const float *g, const float *c, uint64_t *bits_out, uint64_t d, void *stream)
{
    if (g == nullptr || bits_out == nullptr || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(bits_out, 8))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const uint64_t n_words = (d + 63) / 64;
    const uint64_t n_waves = (n_words + kWordsPerWave - 1) / kWordsPerWave;
    hipLaunchKernelGGL(compress_kernel, dim3(blocks_for(n_waves * 64)), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream), g, c, bits_out, d, n_words);
    return finish_launch();
}

static int launch_hop_merge(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                            uint64_t word_begin, uint64_t n_words, uint32_t w_recv, uint32_t w_local,
                            uint32_t hop_id, uint64_t seed, void *stream,
                            const uint64_t *seed_ptr = nullptr)
{
    if (recv == nullptr || local == nullptr || out == nullptr || w_local == 0 ||
        w_recv > 0x7FFFFFFFu || w_local > 0x7FFFFFFFu || n_words > kMaxElements / 64)
        return MARSIT_EINVAL;
    if (!aligned_to(recv, 8) || !aligned_to(local, 8) || !aligned_to(out, 8))
        return MARSIT_EALIGN;
    if (n_words == 0)
        return MARSIT_OK;
    const bool always_local = (w_recv == 0);
    const uint32_t threshold = always_local ? 0xFFFFFFFFu : weighted_threshold(w_recv, w_local);
    hipLaunchKernelGGL(hop_merge_kernel, dim3(blocks_for(n_words * 16)), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint32_t *>(recv),
                       reinterpret_cast<const uint32_t *>(local), reinterpret_cast<uint32_t *>(out),
                       word_begin, n_words, threshold, always_local, hop_id,
                       static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), seed_ptr);
    return finish_launch();
}

int marsit_hop_merge_device_seed(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                                 uint64_t word_begin, uint64_t n_words, uint32_t fold, uint32_t hop_id,
                                 const uint64_t *seed_device, void *stream)
{
    if (fold == 0 || seed_device == nullptr)
        return MARSIT_EINVAL;
    if (!aligned_to(seed_device, 8))
        return MARSIT_EALIGN;
    return launch_hop_merge(recv, local, out, word_begin, n_words, fold - 1, 1, hop_id, 0, stream,
                            seed_device);
}

__global__ void set_seed_kernel(uint64_t *slot, uint64_t seed) { *slot = seed; }

int marsit_set_device_seed(uint64_t *seed_device, uint64_t seed, void *stream)
{
    if (seed_device == nullptr)
        return MARSIT_EINVAL;
    if (!aligned_to(seed_device, 8))
        return MARSIT_EALIGN;
    hipLaunchKernelGGL(set_seed_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), seed_device,
                       seed);
    return finish_launch();
}

int marsit_hop_merge(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                     uint64_t word_begin, uint64_t n_words, uint32_t fold, uint32_t hop_id,
                     uint64_t seed, void *stream)
{
    if (fold == 0)
        return MARSIT_EINVAL;
    return launch_hop_merge(recv, local, out, word_begin, n_words, fold - 1, 1, hop_id, seed, stream);
}

int marsit_hop_merge_weighted(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                              uint64_t word_begin, uint64_t n_words, uint32_t w_recv,
                              uint32_t w_local, uint32_t hop_id, uint64_t seed, void *stream)
{
    return launch_hop_merge(recv, local, out, word_begin, n_words, w_recv, w_local, hop_id, seed, stream);
}

int marsit_decode_compensate(const uint64_t *bits, const float *g, const float *c, float scale,
                             float *update_out, float *c_out, uint64_t d, void *stream)
{
    if (bits == nullptr || g == nullptr || c_out == nullptr || !std::isfinite(scale) ||
        d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(bits, 8) || !aligned_to(g, 4) || !aligned_to(c, 4) ||
        !aligned_to(update_out, 4) || !aligned_to(c_out, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const bool aligned = aligned_to(g, 16) && aligned_to(c, 16) && aligned_to(update_out, 16) &&
                         aligned_to(c_out, 16);
    hipLaunchKernelGGL(decode_compensate_kernel, dim3(blocks_for((d + 3) >> 2)), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint32_t *>(bits), g,
                       c, update_out, c_out, d, float_bits_host(scale), aligned);
    return finish_launch();
}

int marsit_ring_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                         uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                         uint32_t grid_x, void *stream)
{
    if (g == nullptr || c == nullptr || update_out == nullptr || M == 0 ||
        M > MARSIT_MAX_WORKERS || ld < d || !std::isfinite(scale) || d > kMaxElements)
        return MARSIT_EINVAL;
    const uint32_t X = (grid_x == 0) ? M : grid_x;
    if (M % X != 0)
        return MARSIT_EINVAL;
    const uint32_t Y = M / X;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4) ||
        !aligned_to(bits_out, 8))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;

    const uint64_t n_words = (d + 63) / 64;
    uint64_t bounds[MARSIT_MAX_WORKERS + 1];
    split_bounds_host(n_words, M, grid_x, bounds);
    PartTable parts;
    for (uint32_t k = 0; k <= MARSIT_MAX_WORKERS; ++k)
        parts.bound[k] = static_cast<uint32_t>(k <= M ? bounds[k] : n_words);

    const bool aligned = aligned_to(g, 16) && aligned_to(c, 16) && aligned_to(update_out, 16) &&
                         (ld % 4 == 0);
    const uint32_t scale_bits = float_bits_host(scale);
    const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
    uint32_t *bits32 = reinterpret_cast<uint32_t *>(bits_out);
    hipStream_t s = static_cast<hipStream_t>(stream);

    // Whole packed words of an aligned input go to the kernel compiled for this schedule, the
    // ragged last word (and every input without a compiled schedule or with odd alignment) to the
    // generic kernel.  The two write disjoint outputs.
    const SyncLauncher fast = aligned ? find_specialisation(X, Y) : nullptr;
    uint64_t generic_col_begin = 0;
    if (fast != nullptr) {
        const uint64_t fast_cols = (d / 64) * 16;
        if (fast_cols > 0) {
            fast(g, c, update_out, bits32, fast_cols, ld, scale_bits, key0, key1, parts, s);
            const int rc = finish_launch();
            if (rc != MARSIT_OK)
                return rc;
        }
        generic_col_begin = fast_cols;
    }
    const uint64_t n_cols = (d + 3) >> 2;
    if (generic_col_begin < n_cols) {
        ThresholdTable thresholds;
        thresholds.thr[0] = 0;
        thresholds.thr[1] = 0xFFFFFFFFu;
        for (uint32_t m = 2; m <= MARSIT_MAX_WORKERS; ++m)
            thresholds.thr[m] = keep_threshold(m);
        const uint32_t blocks =
            static_cast<uint32_t>((n_cols - generic_col_begin + kSyncBlock - 1) / kSyncBlock);
        if (M <= kMaxStagedWorkers)
            hipLaunchKernelGGL(sync_step_generic_kernel<true>, dim3(blocks), dim3(kSyncBlock),
                               generic_lds_bytes(M), s, g, c, update_out, bits32, d, ld,
                               generic_col_begin, scale_bits, key0, key1, X, Y, aligned, parts, thresholds);
        else
            hipLaunchKernelGGL(sync_step_generic_kernel<false>, dim3(blocks), dim3(kSyncBlock), 0, s, g, c,
                               update_out, bits32, d, ld, generic_col_begin, scale_bits, key0, key1, X, Y,
                               aligned, parts, thresholds);
        return finish_launch();
    }
    return MARSIT_OK;
}

int marsit_tree_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                         uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed, void *stream)
{
    if (g == nullptr || c == nullptr || update_out == nullptr || M == 0 ||
        M > MARSIT_MAX_WORKERS || ld < d || !std::isfinite(scale) || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4) ||
        !aligned_to(bits_out, 8))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const bool aligned = aligned_to(g, 16) && aligned_to(c, 16) && aligned_to(update_out, 16) &&
                         (ld % 4 == 0);
    const uint32_t scale_bits = float_bits_host(scale);
    const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
    uint32_t *bits32 = reinterpret_cast<uint32_t *>(bits_out);
    hipStream_t s = static_cast<hipStream_t>(stream);

    const TreeLauncher fast = aligned ? find_tree(M) : nullptr;
    uint64_t generic_col_begin = 0;
    if (fast != nullptr) {
        const uint64_t fast_cols = (d / 64) * 16;
        if (fast_cols > 0) {
            fast(g, c, update_out, bits32, fast_cols, ld, scale_bits, key0, key1, s);
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
        const uint32_t blocks =
            static_cast<uint32_t>((n_cols - generic_col_begin + kSyncBlock - 1) / kSyncBlock);
        if (M <= kMaxStagedWorkers)
            hipLaunchKernelGGL(tree_step_generic_kernel<true>, dim3(blocks), dim3(kSyncBlock),
                               generic_lds_bytes(M), s, g, c, update_out, bits32, d, ld,
                               generic_col_begin, scale_bits, key0, key1, M, top_level, aligned);
        else
            hipLaunchKernelGGL(tree_step_generic_kernel<false>, dim3(blocks), dim3(kSyncBlock), 0, s, g, c,
                               update_out, bits32, d, ld, generic_col_begin, scale_bits, key0, key1, M,
                               top_level, aligned);
        return finish_launch();
    }
    return MARSIT_OK;
}

uint64_t marsit_chain_workspace_words(uint32_t M, uint64_t d, uint32_t grid_x)
{
    if (M == 0 || M > MARSIT_MAX_WORKERS || d > kMaxElements)
        return 0;
    const uint32_t X = (grid_x == 0) ? M : grid_x;
    if (M % X != 0)
        return 0;
    const uint32_t Y = M / X;
    const uint64_t n_words = (d + 63) / 64;
    return (static_cast<uint64_t>(M) + (Y > 1 ? Y : 0)) * n_words;
}

int marsit_chain_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                          uint64_t *workspace, uint32_t M, uint64_t d, uint64_t ld, float scale,
                          uint64_t seed, uint32_t grid_x, void *stream)
{
    if (g == nullptr || c == nullptr || update_out == nullptr || bits_out == nullptr ||
        workspace == nullptr || M == 0 || M > MARSIT_MAX_WORKERS || ld < d || !std::isfinite(scale) ||
        d > kMaxElements)
        return MARSIT_EINVAL;
    const uint32_t X = (grid_x == 0) ? M : grid_x;
    if (M % X != 0)
        return MARSIT_EINVAL;
    const uint32_t Y = M / X;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4) ||
        !aligned_to(bits_out, 8) || !aligned_to(workspace, 8))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;

    const uint64_t W = (d + 63) / 64;
    uint64_t fine[MARSIT_MAX_WORKERS + 1];
    split_bounds_host(W, M, grid_x, fine);
    uint64_t *maps = workspace;                    // [M][W]  every worker's own signs
    uint64_t *rows = workspace + static_cast<size_t>(M) * W;   // [Y][W]  row results (torus)
    int rc;

    for (uint32_t m = 0; m < M; ++m) {
        rc = marsit_compress(g + static_cast<size_t>(m) * ld, c + static_cast<size_t>(m) * ld,
                             maps + static_cast<size_t>(m) * W, d, stream);
        if (rc != MARSIT_OK)
            return rc;
    }

    // row phase: row-part a = words [fine[a*Y], fine[(a+1)*Y]); in row y its chain starts at column a.
    // The first holder sends its own signs (fold 1 copies them), every later hop h folds column (a+h) mod X.
    for (uint32_t a = 0; a < X; ++a) {
        const uint64_t lo = fine[a * Y], n = fine[(a + 1) * Y] - lo;
        if (n == 0)
            continue;
        for (uint32_t y = 0; y < Y; ++y) {
            uint64_t *r = (Y > 1 ? rows + static_cast<size_t>(y) * W : bits_out) + lo;
            const uint64_t *first = maps + static_cast<size_t>(y * X + a) * W + lo;
            rc = marsit_hop_merge(first, first, r, lo, n, 1, 0, seed, stream);
            if (rc != MARSIT_OK)
                return rc;
            for (uint32_t h = 1; h < X; ++h) {
                const uint64_t *local = maps + static_cast<size_t>(y * X + (a + h) % X) * W + lo;
                rc = marsit_hop_merge(r, local, r, lo, n, h + 1, row_hop_id(y, h), seed, stream);
                if (rc != MARSIT_OK)
                    return rc;
            }
        }
    }
    // column phase over the row results: sub-part b of row-part a starts at row b
    if (Y > 1) {
        for (uint32_t f = 0; f < M; ++f) {
            const uint32_t b = f % Y;
            const uint64_t lo = fine[f], n = fine[f + 1] - lo;
            if (n == 0)
                continue;
            uint64_t *r = bits_out + lo;
            const uint64_t *first = rows + static_cast<size_t>(b) * W + lo;
            rc = marsit_hop_merge(first, first, r, lo, n, 1, 0, seed, stream);
            if (rc != MARSIT_OK)
                return rc;
            for (uint32_t k = 1; k < Y; ++k) {
                const uint64_t *local = rows + static_cast<size_t>((b + k) % Y) * W + lo;
                rc = marsit_hop_merge(r, local, r, lo, n, k + 1, col_hop_id(k), seed, stream);
                if (rc != MARSIT_OK)
                    return rc;
            }
        }
    }

    for (uint32_t m = 0; m < M; ++m) {
        rc = marsit_decode_compensate(bits_out, g + static_cast<size_t>(m) * ld,
                                      c + static_cast<size_t>(m) * ld, scale,
                                      m == 0 ? update_out : nullptr, c + static_cast<size_t>(m) * ld,
                                      d, stream);
        if (rc != MARSIT_OK)
            return rc;
    }
    return MARSIT_OK;
}

int marsit_full_sync(const float *g, float *c, float *update_out, uint32_t M, uint64_t d,
                     uint64_t ld, void *stream)
{
    if (g == nullptr || c == nullptr || update_out == nullptr || M == 0 ||
        M > MARSIT_MAX_WORKERS || ld < d || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const bool aligned = aligned_to(g, 16) && aligned_to(c, 16) && aligned_to(update_out, 16) &&
                         (ld % 4 == 0);
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint64_t col_begin = 0;
    const FullSyncLauncher fast = aligned ? find_full_sync(M) : nullptr;
    if (fast != nullptr && d >= 4) {
        col_begin = d / 4;
        fast(g, c, update_out, col_begin, ld, s);
        const int rc = finish_launch();
        if (rc != MARSIT_OK)
            return rc;
    }
    const uint64_t n_cols = (d + 3) >> 2;
    if (col_begin < n_cols) {
        hipLaunchKernelGGL(full_sync_kernel, dim3(blocks_for(n_cols - col_begin)), dim3(kBlock), 0, s,
                           g, c, update_out, M, d, ld, col_begin, aligned);
        return finish_launch();
    }
    return MARSIT_OK;
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

static int launch_vote(int mode, const float *g, const float *c, uint64_t *bits_out, uint32_t M,
                       uint64_t d, uint64_t ld, void *stream)
{
    if (g == nullptr || c == nullptr || bits_out == nullptr || M == 0 || M > MARSIT_MAX_WORKERS ||
        ld < d || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(bits_out, 8))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const bool aligned = aligned_to(g, 16) && aligned_to(c, 16) && (ld % 4 == 0);
    const dim3 grid(blocks_for((d + 3) >> 2)), block(kBlock);
    uint32_t *bits32 = reinterpret_cast<uint32_t *>(bits_out);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mode == kAggregateSign)
        hipLaunchKernelGGL(vote_kernel<kAggregateSign>, grid, block, 0, s, g, c, bits32, M, d, ld, aligned);
    else
        hipLaunchKernelGGL(vote_kernel<kMajorityVote>, grid, block, 0, s, g, c, bits32, M, d, ld, aligned);
    return finish_launch();
}

int marsit_aggregate_sign(const float *g, const float *c, uint64_t *bits_out, uint32_t M, uint64_t d,
                          uint64_t ld, void *stream)
{
    return launch_vote(kAggregateSign, g, c, bits_out, M, d, ld, stream);
}

int marsit_majority_vote(const float *g, const float *c, uint64_t *bits_out, uint32_t M, uint64_t d,
                         uint64_t ld, void *stream)
{
    return launch_vote(kMajorityVote, g, c, bits_out, M, d, ld, stream);
}

int marsit_count_matching(const uint64_t *bits_a, const uint64_t *bits_b, uint64_t d,
                          uint64_t *count_out, void *stream)
{
    if (bits_a == nullptr || bits_b == nullptr || count_out == nullptr || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(bits_a, 8) || !aligned_to(bits_b, 8) || !aligned_to(count_out, 8))
        return MARSIT_EALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned long long *count = reinterpret_cast<unsigned long long *>(count_out);
    hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(1), 0, s, count);
    int rc = finish_launch();
    if (rc != MARSIT_OK || d == 0)
        return rc;
    const uint64_t n_words = (d + 63) / 64;
    hipLaunchKernelGGL(count_matching_kernel, dim3(blocks_for(n_words)), dim3(kBlock), 0, s, bits_a,
                       bits_b, d, n_words, count);
    return finish_launch();
}

int marsit_ssdm_cascade_hop(const uint64_t *recv_bits, const float *recv_norm, const float *g,
                            const float *c, uint64_t *bits_out, float *norm_out, void *workspace,
                            uint64_t word_begin, uint64_t n, uint32_t hop_id, uint64_t seed,
                            void *stream)
{
    if (g == nullptr || c == nullptr || bits_out == nullptr || norm_out == nullptr ||
        workspace == nullptr || (recv_bits != nullptr && recv_norm == nullptr) ||
        (recv_norm != nullptr && recv_norm == norm_out) || n > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(bits_out, 8) ||
        !aligned_to(recv_bits, 8) || !aligned_to(norm_out, 4) || !aligned_to(recv_norm, 4) ||
        !aligned_to(workspace, 8))
        return MARSIT_EALIGN;
    if (n == 0)
        return MARSIT_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool aligned = aligned_to(g, 16) && aligned_to(c, 16);
    const uint64_t n_cols = (n + 3) >> 2;
    uint32_t n_partials = blocks_for(n_cols);
    if (n_partials > kCascadeMaxPartials)
        n_partials = kCascadeMaxPartials;
    double *partial = static_cast<double *>(workspace);
    const uint32_t *recv32 = reinterpret_cast<const uint32_t *>(recv_bits);
    hipLaunchKernelGGL(cascade_norm_partial_kernel, dim3(n_partials), dim3(kBlock), 0, s, recv32,
                       recv_norm, g, c, n, aligned, partial);
    int rc = finish_launch();
    if (rc != MARSIT_OK)
        return rc;
    hipLaunchKernelGGL(cascade_norm_final_kernel, dim3(1), dim3(1), 0, s, partial, n_partials, norm_out,
                       static_cast<float *>(nullptr));
    rc = finish_launch();
    if (rc != MARSIT_OK)
        return rc;
    hipLaunchKernelGGL(cascade_sign_kernel, dim3(blocks_for(n_cols)), dim3(kBlock), 0, s, recv32, recv_norm,
                       g, c, norm_out, reinterpret_cast<uint32_t *>(bits_out), n, word_begin, hop_id,
                       static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), aligned);
    return finish_launch();
}

int marsit_cascade_ring_step_sim(const float *g, const float *c, float *update_out, uint64_t *bits_out,
                                 float *norms_out, void *workspace, uint32_t M, uint64_t d, uint64_t ld,
                                 uint64_t seed, void *stream)
{
    if (g == nullptr || c == nullptr || update_out == nullptr || bits_out == nullptr ||
        norms_out == nullptr || workspace == nullptr || M == 0 || M > MARSIT_MAX_WORKERS || ld < d ||
        d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(update_out, 4) ||
        !aligned_to(bits_out, 8) || !aligned_to(norms_out, 4) || !aligned_to(workspace, 8))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const uint64_t W = (d + 63) / 64;
    uint64_t bound[MARSIT_MAX_WORKERS + 1];
    split_bounds_host(W, M, 0, bound);
    // workspace: the partial sums, then two norm slots used in turn by the hops of a chain
    float *norm_slot = reinterpret_cast<float *>(static_cast<double *>(workspace) + kCascadeMaxPartials);
    hipStream_t s = static_cast<hipStream_t>(stream);

    for (uint32_t i = 0; i < M; ++i) {
        const uint64_t lo = bound[i], hi = bound[i + 1];
        if (hi == lo)
            continue;
        const uint64_t e0 = lo * 64, e1 = (hi * 64 < d) ? hi * 64 : d, n = e1 - e0;
        uint64_t *bits = bits_out + lo;                    // the chain is carried in place
        for (uint32_t h = 0; h < M; ++h) {
            const uint32_t worker = (i + h) % M;
            float *norm_new = (h == M - 1) ? norms_out + i : norm_slot + (h & 1u);
            const float *norm_prev = (h == 0) ? nullptr : norm_slot + ((h - 1) & 1u);
            const int rc = marsit_ssdm_cascade_hop(h == 0 ? nullptr : bits, norm_prev,
                                                   g + static_cast<size_t>(worker) * ld + e0,
                                                   c + static_cast<size_t>(worker) * ld + e0, bits,
                                                   norm_new, workspace, lo, n, (3u << 16) | h, seed, s);
            if (rc != MARSIT_OK)
                return rc;
        }
        hipLaunchKernelGGL(cascade_decode_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, s,
                           reinterpret_cast<const uint32_t *>(bits), norms_out + i, update_out + e0, n,
                           static_cast<float>(M));
        const int rc = finish_launch();
        if (rc != MARSIT_OK)
            return rc;
    }
    return MARSIT_OK;
}

int marsit_apply_update(float *x, const float *update, uint64_t d, void *stream)
{
    if (x == nullptr || update == nullptr || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(update, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const bool aligned = aligned_to(x, 16) && aligned_to(update, 16);
    hipLaunchKernelGGL(apply_update_kernel, dim3(blocks_for((d + 3) >> 2)), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream), x, update, d, aligned);
    return finish_launch();
}

}   // extern "C"
