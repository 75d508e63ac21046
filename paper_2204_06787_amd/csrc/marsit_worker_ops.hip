// Per-worker kernels of the Marsit one-bit pass (compress, one hop of the merge, decode and
// compensate, model update), the hop-by-hop chain built from them, and the host-side utilities of
// the C ABI.

#include "marsit_device.hpp"
#include "marsit_host.hpp"

#include <atomic>

namespace marsit {

thread_local int tls_last_hip_error = 0;

// Workspace of marsit_exchange_step_sim_static.  Every GPU the library runs on holds its own copy
// of this array, at its own address, until the process ends.  In host code the name is only a
// handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) uint64_t scratch[MARSIT_STATIC_SCRATCH_WORDS];

constexpr int kMaxDevices = 64;
static std::atomic<uint64_t *> scratch_address[kMaxDevices];

// Device address of `scratch` on the current device; resolved on the first call per device.
static int static_scratch_address(uint64_t **out)
{
    int device = -1;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess) {
        tls_last_hip_error = static_cast<int>(err);
        return MARSIT_EHIP;
    }
    if (device < 0 || device >= kMaxDevices)
        return MARSIT_EINVAL;
    uint64_t *ptr = scratch_address[device].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        void *resolved = nullptr;
        err = hipGetSymbolAddress(&resolved, HIP_SYMBOL(scratch));
        if (err != hipSuccess || resolved == nullptr) {
            tls_last_hip_error = static_cast<int>(err);
            return MARSIT_EHIP;
        }
        ptr = static_cast<uint64_t *>(resolved);
        scratch_address[device].store(ptr, std::memory_order_release);   // same value from any thread
    }
    *out = ptr;
    return MARSIT_OK;
}

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
// marsit_compress_hop_merge and marsit_compress: the sign step and one merge in one pass.  lane =
// one column of 4 elements = nibble q of packed word i: the local nibble comes from the sign bits
// of g + c instead of a stored bitmap, the rest is hop_merge_kernel; the nibbles of a word are
// OR-gathered over the half rows with DPP moves.  With fold count 1 (marsit_compress, or the first
// holder of a part) nothing is received and nothing is drawn.
// -------------------------------------------------------------------------------------------------
// Launch shape of the kernels that stream one worker's vectors: one-wavefront workgroups, every lane
// takes COLS columns 64 apart (so each access of the wavefront is one contiguous KB), all of a
// lane's loads are issued before the first use, non-temporal accesses.  With two to five streams
// these kernels want every wavefront the CU can hold (measured at 25.6 M elements: one column per
// lane 80-82 % of the HBM peak for decode, model update and momentum, 74-77 % with four; two
// columns per lane for the sign step, 79 % against 76 %).
constexpr int kCompressCols = 2;                      // sign step (with or without a merge)
constexpr int kStreamCols = 1;                        // decode, model update, momentum

inline uint32_t stream_blocks(uint64_t n_cols, int cols_per_lane)
{
    const uint64_t per_block = static_cast<uint64_t>(kSyncBlock) * static_cast<uint64_t>(cols_per_lane);
    return static_cast<uint32_t>((n_cols + per_block - 1) / per_block);
}

template <int COLS>
__global__ void __launch_bounds__(kSyncBlock)
compress_hop_merge_kernel(const uint32_t *recv32, const float *__restrict__ g,
                          const float *__restrict__ c, uint32_t *out32, uint64_t word_begin,
                          uint64_t n, uint32_t threshold, bool always_local, uint32_t hop_id,
                          uint32_t key0, uint32_t key1)
{
    const uint64_t n_cols = (n + 3) >> 2;
    const uint64_t n_words = (n + 63) >> 6;
    const uint64_t col0 = static_cast<uint64_t>(blockIdx.x) * (kSyncBlock * COLS) + threadIdx.x;
    const uint32_t q = threadIdx.x & 15u;
    const uint32_t shift = (q & 7u) * 4u;
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};

    f32x4 gv[COLS], cv[COLS];
    uint32_t rv[COLS];
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        gv[k] = zero;
        cv[k] = zero;
        rv[k] = 0;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= n;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(n - e);
            gv[k] = load4<true>(g + e, full, n_valid);
            if (c != nullptr)
                cv[k] = load4<true>(c + e, full, n_valid);
            if (!always_local)
                rv[k] = recv32[2u * static_cast<size_t>(col >> 4) + (q >> 3)];
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        const uint64_t i = col >> 4;
        uint32_t nib = 0;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const uint32_t n_valid = (e + 4 <= n) ? 4u : static_cast<uint32_t>(n - e);
            const f32x4 sv = gv[k] + cv[k];
            uint32_t l = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                l |= (static_cast<uint32_t>(j) < n_valid && (f32_bits(sv[j]) >> 31) == 0u) ? (1u << j) : 0u;
            const uint32_t r = (rv[k] >> shift) & 0xFu;
            uint32_t t = 0xFu;                                    // fold 1: the local signs as they are
            if (!always_local) {
                const uint64_t w = word_begin + i;
                uint32_t u[4];
                philox4x32_10(q, hop_id, static_cast<uint32_t>(w), static_cast<uint32_t>(w >> 32), key0,
                              key1, u);
                t = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    t |= (u[j] < threshold) ? (1u << j) : 0u;
            }
            nib = (r ^ ((r ^ l) & t)) & ((1u << n_valid) - 1u);   // t ? l : r; bits past the end stay 0
        }
        const uint32_t half = half_row_or(nib << shift);           // every lane takes part
        if (i < n_words && (q & 7u) == 0u)
            out32[2u * static_cast<size_t>(i) + (q >> 3)] = half;
    }
}

// -------------------------------------------------------------------------------------------------
// marsit_fold_segments: the whole chain of a part in one launch, for the owner of the part that has
// received the K sign segments (all-to-all exchange instead of K-1 ring hops).  lane = (packed
// word i, nibble q) as in hop_merge_kernel.  The draws do not depend on the data: per bit, the last
// hop whose draw succeeds names the operand whose sign survives; then each operand's nibble is
// read once and selected.  Same draws, same result as K-1 marsit_hop_merge launches.
// -------------------------------------------------------------------------------------------------
struct FoldThresholds {
    uint32_t thr[MARSIT_MAX_WORKERS + 1];     // thr[m] = floor(2^32 / m)
};

__global__ void __launch_bounds__(kBlock)
fold_segments_kernel(const uint32_t *__restrict__ maps32, uint64_t stride_halves, uint32_t K,
                     uint32_t first, uint32_t *__restrict__ out32, uint64_t word_begin,
                     uint64_t n_words, uint32_t hop_base, uint32_t key0, uint32_t key1,
                     FoldThresholds thresholds)
{
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    const uint64_t i = col >> 4;
    const uint32_t q = static_cast<uint32_t>(col) & 15u;
    const size_t half_index = 2u * static_cast<size_t>(i) + (q >> 3);
    const uint32_t shift = (q & 7u) * 4u;
    uint32_t nib = 0;

    if (i < n_words) {
        const uint64_t w = word_begin + i;
        uint32_t pick[4] = {0, 0, 0, 0};
        for (uint32_t h = 1; h < K; ++h) {
            uint32_t u[4];
            philox4x32_10(q, hop_base | h, static_cast<uint32_t>(w), static_cast<uint32_t>(w >> 32),
                          key0, key1, u);
            const uint32_t thr = thresholds.thr[h + 1];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                pick[j] = (u[j] < thr) ? h : pick[j];
        }
        uint32_t k = first;
        for (uint32_t h = 0; h < K; ++h) {
            const uint32_t v = (maps32[static_cast<size_t>(k) * stride_halves + half_index] >> shift) & 0xFu;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                nib = (pick[j] == h) ? ((nib & ~(1u << j)) | (v & (1u << j))) : nib;
            k = (k + 1 == K) ? 0u : k + 1;
        }
    }

    const uint32_t half = half_row_or(nib << shift);
    if (i < n_words && (q & 7u) == 0u)
        out32[half_index] = half;
}

// -------------------------------------------------------------------------------------------------
// marsit_decode_compensate: lane = one column of 4 elements.
// -------------------------------------------------------------------------------------------------
template <int COLS>
__global__ void __launch_bounds__(kSyncBlock)
decode_compensate_kernel(const uint32_t *__restrict__ bits32, const float *__restrict__ g,
                         const float *c, float *__restrict__ update, float *c_out, uint64_t d,
                         uint32_t scale_bits, float *__restrict__ x_model)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col0 = static_cast<uint64_t>(blockIdx.x) * (kSyncBlock * COLS) + threadIdx.x;
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};

    f32x4 gv[COLS], cv[COLS], xv[COLS];
    uint32_t bv[COLS];
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        gv[k] = zero;
        cv[k] = zero;
        xv[k] = zero;
        bv[k] = 0;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= d;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
            gv[k] = load4(g + e, full, n_valid);
            if (c != nullptr)
                cv[k] = load4(c + e, full, n_valid);
            if (x_model != nullptr)
                xv[k] = load4(x_model + e, full, n_valid);
            bv[k] = bits32[col >> 3];
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= d;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
            const uint32_t nib = (bv[k] >> ((static_cast<uint32_t>(col) & 7u) * 4u)) & 0xFu;
            const f32x4 sv = gv[k] + cv[k];
            f32x4 upd;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                upd[j] = __uint_as_float(scale_bits ^ (((nib >> j) & 1u) ? 0u : 0x80000000u));
            if (update != nullptr)
                store4<MARSIT_STREAMING_STORES>(update + e, upd, full, n_valid);
            if (x_model != nullptr)      // Algorithm 2, model update in the same pass
                store4<MARSIT_STREAMING_STORES>(x_model + e, xv[k] - upd, full, n_valid);
            store4<MARSIT_STREAMING_STORES>(c_out + e, sv - upd, full, n_valid);
        }
    }
}

template <int COLS>
__global__ void __launch_bounds__(kSyncBlock)
apply_update_kernel(float *__restrict__ x, const float *__restrict__ update, uint64_t d)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col0 = static_cast<uint64_t>(blockIdx.x) * (kSyncBlock * COLS) + threadIdx.x;
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4 xv[COLS], uv[COLS];
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        xv[k] = zero;
        uv[k] = zero;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= d;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
            xv[k] = load4<true>(x + e, full, n_valid);
            uv[k] = load4<true>(update + e, full, n_valid);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= d;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
            store4<MARSIT_STREAMING_STORES>(x + e, xv[k] - uv[k], full, n_valid);
        }
    }
}

// Local heavy-ball momentum for all workers in one launch (blockIdx.y = worker):
// buf <- beta * buf + grad; g <- eta_l * buf.  Three separately rounded fp32 operations (the library
// is built without contraction).  g may be the same array as grad: a lane reads its elements
// before it writes them.
template <int COLS>
__global__ void __launch_bounds__(kSyncBlock)
local_momentum_kernel(float *__restrict__ buf, const float *grad, float *g_out, uint64_t d,
                      uint64_t ld, float beta, float eta_l)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col0 = static_cast<uint64_t>(blockIdx.x) * (kSyncBlock * COLS) + threadIdx.x;
    const size_t row = static_cast<size_t>(blockIdx.y) * ld;
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4 bv[COLS], gv[COLS];
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        bv[k] = zero;
        gv[k] = zero;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= d;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
            bv[k] = load4<true>(buf + row + e, full, n_valid);
            gv[k] = load4<true>(grad + row + e, full, n_valid);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= d;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
            const f32x4 carried = bv[k] * beta;
            const f32x4 v = carried + gv[k];
            store4<true>(buf + row + e, v, full, n_valid);
            store4<true>(g_out + row + e, v * eta_l, full, n_valid);
        }
    }
}

// Local Adam for all workers in one launch (blockIdx.y = worker), the published form with bias
// correction (Section 5 of the paper names the optimizer only):
//   p <- beta1 * p + (1 - beta1) * a;   q <- beta2 * q + (1 - beta2) * (a * a);
//   g <- eta_l * ((p / bias1) / (sqrt(q / bias2) + eps)).
// One fp32 rounding per operation in this order (the library is built without contraction, and
// hipcc's fp32 division and square root are correctly rounded).  rest1 = 1 - beta1 and
// rest2 = 1 - beta2 are rounded once on the host.  g may be the same array as the gradient: a lane
// reads its elements before it writes them.
template <int COLS>
__global__ void __launch_bounds__(kSyncBlock)
local_adam_kernel(float *__restrict__ mom1, float *__restrict__ mom2, const float *grad, float *g_out,
                  uint64_t d, uint64_t ld, float beta1, float rest1, float beta2, float rest2, float eps,
                  float eta_l, float bias1, float bias2)
{
    const uint64_t n_cols = (d + 3) >> 2;
    const uint64_t col0 = static_cast<uint64_t>(blockIdx.x) * (kSyncBlock * COLS) + threadIdx.x;
    const size_t row = static_cast<size_t>(blockIdx.y) * ld;
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4 pv[COLS], qv[COLS], av[COLS];
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        pv[k] = zero;
        qv[k] = zero;
        av[k] = zero;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= d;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
            pv[k] = load4<true>(mom1 + row + e, full, n_valid);
            qv[k] = load4<true>(mom2 + row + e, full, n_valid);
            av[k] = load4<true>(grad + row + e, full, n_valid);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < COLS; ++k) {
        const uint64_t col = col0 + static_cast<uint64_t>(k) * kSyncBlock;
        if (col < n_cols) {
            const uint64_t e = col << 2;
            const bool full = e + 4 <= d;
            const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(d - e);
            const f32x4 p_old = pv[k] * beta1;
            const f32x4 p_new = av[k] * rest1;
            const f32x4 p = p_old + p_new;
            const f32x4 a2 = av[k] * av[k];
            const f32x4 q_old = qv[k] * beta2;
            const f32x4 q_new = a2 * rest2;
            const f32x4 q = q_old + q_new;
            f32x4 step;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float p_hat = p[j] / bias1;
                const float q_hat = q[j] / bias2;
                const float denom = sqrtf(q_hat) + eps;
                const float dir = p_hat / denom;
                step[j] = eta_l * dir;
            }
            store4<true>(mom1 + row + e, p, full, n_valid);
            store4<true>(mom2 + row + e, q, full, n_valid);
            store4<true>(g_out + row + e, step, full, n_valid);
        }
    }
}

}   // namespace marsit

using namespace marsit;

extern "C" {

int marsit_version(void) { return 210; }

int marsit_last_hip_error(void) { return tls_last_hip_error; }

const char *marsit_status_string(int status)
{
    switch (status) {
    case MARSIT_OK: return "ok";
    case MARSIT_EINVAL: return "invalid argument";
    case MARSIT_EALIGN: return "pointer not aligned to its element size";
    case MARSIT_EHIP: return "HIP call failed (see marsit_last_hip_error)";
    case MARSIT_ESCRATCH: return "input needs more workspace than the library's static scratch array holds";
    default: return "unknown status";
    }
}

uint64_t marsit_grid_work_items(uint64_t d)
{
    if (d == 0 || d > kMaxElements)
        return 0;
    return static_cast<uint64_t>(blocks_for((d + 3) >> 2)) * kBlock;
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
    // the sign step alone is the sign-and-merge kernel with fold count 1: nothing received, no draw
    const uint64_t n_words = (d + 63) / 64;
    hipLaunchKernelGGL(compress_hop_merge_kernel<kCompressCols>, dim3(stream_blocks(n_words * 16, kCompressCols)),
                       dim3(kSyncBlock), 0, static_cast<hipStream_t>(stream), static_cast<const uint32_t *>(nullptr),
                       g, c, reinterpret_cast<uint32_t *>(bits_out), 0, d, 0xFFFFFFFFu, true, 0u, 0u, 0u);
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

int marsit_compress_hop_merge(const uint64_t *recv, const float *g, const float *c, uint64_t *out,
                              uint64_t word_begin, uint64_t n, uint32_t fold, uint32_t hop_id,
                              uint64_t seed, void *stream)
{
    if (g == nullptr || out == nullptr || fold == 0 || (recv == nullptr && fold != 1) ||
        n > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(recv, 8) || !aligned_to(g, 4) || !aligned_to(c, 4) || !aligned_to(out, 8))
        return MARSIT_EALIGN;
    if (n == 0)
        return MARSIT_OK;
    const bool always_local = (fold == 1);
    const uint32_t threshold = always_local ? 0xFFFFFFFFu : keep_threshold(fold);
    const uint64_t n_words = (n + 63) / 64;
    hipLaunchKernelGGL(compress_hop_merge_kernel<kCompressCols>, dim3(stream_blocks(n_words * 16, kCompressCols)), dim3(kSyncBlock), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint32_t *>(recv), g, c,
                       reinterpret_cast<uint32_t *>(out), word_begin, n, threshold, always_local, hop_id,
                       static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
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

static int decode_impl(const uint64_t *bits, const float *g, const float *c, float scale,
                       float *update_out, float *c_out, float *x_model, uint64_t d, void *stream)
{
    if (bits == nullptr || g == nullptr || c_out == nullptr || !std::isfinite(scale) ||
        d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(bits, 8) || !aligned_to(g, 4) || !aligned_to(c, 4) ||
        !aligned_to(update_out, 4) || !aligned_to(c_out, 4) || !aligned_to(x_model, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    hipLaunchKernelGGL(decode_compensate_kernel<kStreamCols>, dim3(stream_blocks((d + 3) >> 2, kStreamCols)), dim3(kSyncBlock), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint32_t *>(bits), g,
                       c, update_out, c_out, d, float_bits_host(scale), x_model);
    return finish_launch();
}

int marsit_decode_compensate(const uint64_t *bits, const float *g, const float *c, float scale,
                             float *update_out, float *c_out, uint64_t d, void *stream)
{
    return decode_impl(bits, g, c, scale, update_out, c_out, nullptr, d, stream);
}

int marsit_decode_compensate_apply(const uint64_t *bits, const float *g, const float *c, float scale,
                                   float *x, float *update_out, float *c_out, uint64_t d, void *stream)
{
    if (x == nullptr || x == update_out || x == c_out)
        return MARSIT_EINVAL;
    return decode_impl(bits, g, c, scale, update_out, c_out, x, d, stream);
}

int marsit_fold_segments(const uint64_t *maps, uint64_t stride_words, uint32_t K, uint32_t first,
                         uint64_t *out, uint64_t word_begin, uint64_t n_words, uint32_t hop_base,
                         uint64_t seed, void *stream)
{
    if (maps == nullptr || out == nullptr || K == 0 || K > MARSIT_MAX_WORKERS || first >= K ||
        n_words > kMaxElements / 64 || (K > 1 && stride_words < n_words) || (hop_base & 0xFFu) != 0)
        return MARSIT_EINVAL;
    if (!aligned_to(maps, 8) || !aligned_to(out, 8))
        return MARSIT_EALIGN;
    if (n_words == 0)
        return MARSIT_OK;
    FoldThresholds thresholds;
    thresholds.thr[0] = 0;
    thresholds.thr[1] = 0xFFFFFFFFu;
    for (uint32_t m = 2; m <= MARSIT_MAX_WORKERS; ++m)
        thresholds.thr[m] = keep_threshold(m);
    hipLaunchKernelGGL(fold_segments_kernel, dim3(blocks_for(n_words * 16)), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint32_t *>(maps),
                       2u * stride_words, K, first, reinterpret_cast<uint32_t *>(out), word_begin, n_words,
                       hop_base, static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), thresholds);
    return finish_launch();
}

// The one-bit pass as one exchange step: every worker computes its signs, the owner of a part gets
// all K segments of that part (on one GPU they are simply in memory) and folds them in one launch,
// every worker decodes.  Rows first, then columns, on a torus.  Workspace as in marsit_chain_step_sim:
// every word of it that is read has been written earlier in the same call (the M bitmaps by the
// compress launches, the row results by the row folds), so its previous contents do not matter.
static int exchange_step_impl(const float *g, float *c, float *update_out, uint64_t *bits_out,
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
    uint64_t *maps = workspace;                                  // [M][W]  every worker's own signs
    uint64_t *rows = workspace + static_cast<size_t>(M) * W;     // [Y][W]  row results (torus)
    int rc;

    for (uint32_t m = 0; m < M; ++m) {
        rc = marsit_compress(g + static_cast<size_t>(m) * ld, c + static_cast<size_t>(m) * ld,
                             maps + static_cast<size_t>(m) * W, d, stream);
        if (rc != MARSIT_OK)
            return rc;
    }
    // row phase: the owner of row-part a in row y folds the X segments of its row, chain from column a
    for (uint32_t a = 0; a < X; ++a) {
        const uint64_t lo = fine[a * Y], n = fine[(a + 1) * Y] - lo;
        for (uint32_t y = 0; y < Y && n > 0; ++y) {
            uint64_t *r = (Y > 1 ? rows + static_cast<size_t>(y) * W : bits_out) + lo;
            rc = marsit_fold_segments(maps + static_cast<size_t>(y * X) * W + lo, W, X, a, r, lo, n,
                                      row_hop_id(y, 0), seed, stream);
            if (rc != MARSIT_OK)
                return rc;
        }
    }
    // column phase: the owner of sub-part b of row-part a folds the Y row results, chain from row b
    if (Y > 1) {
        for (uint32_t f = 0; f < M; ++f) {
            const uint64_t lo = fine[f], n = fine[f + 1] - lo;
            if (n == 0)
                continue;
            rc = marsit_fold_segments(rows + lo, W, Y, f % Y, bits_out + lo, lo, n, col_hop_id(0), seed,
                                      stream);
            if (rc != MARSIT_OK)
                return rc;
        }
    }
    for (uint32_t m = 0; m < M; ++m) {
        rc = marsit_decode_compensate(bits_out, g + static_cast<size_t>(m) * ld,
                                      c + static_cast<size_t>(m) * ld, scale,
                                      m == 0 ? update_out : nullptr, c + static_cast<size_t>(m) * ld, d,
                                      stream);
        if (rc != MARSIT_OK)
            return rc;
    }
    return MARSIT_OK;
}

int marsit_exchange_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                             uint64_t *workspace, uint32_t M, uint64_t d, uint64_t ld, float scale,
                             uint64_t seed, uint32_t grid_x, void *stream)
{
    return exchange_step_impl(g, c, update_out, bits_out, workspace, M, d, ld, scale, seed, grid_x, stream);
}

// marsit_exchange_step_sim for callers that cannot allocate: the workspace is the library's own
// static array.  Its device address is looked up once per device (the first call there) and kept.
int marsit_exchange_step_sim_static(const float *g, float *c, float *update_out, uint64_t *bits_out,
                                    uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                                    uint32_t grid_x, void *stream)
{
    // argument errors first, so that they read the same as marsit_exchange_step_sim's
    if (g == nullptr || c == nullptr || update_out == nullptr || bits_out == nullptr || M == 0 ||
        M > MARSIT_MAX_WORKERS || ld < d || !std::isfinite(scale) || d > kMaxElements ||
        (grid_x != 0 && M % grid_x != 0))
        return MARSIT_EINVAL;
    if (marsit_chain_workspace_words(M, d, grid_x) > MARSIT_STATIC_SCRATCH_WORDS)
        return MARSIT_ESCRATCH;
    uint64_t *workspace = nullptr;
    const int rc = static_scratch_address(&workspace);
    if (rc != MARSIT_OK)
        return rc;
    return exchange_step_impl(g, c, update_out, bits_out, workspace, M, d, ld, scale, seed, grid_x, stream);
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

int marsit_apply_update(float *x, const float *update, uint64_t d, void *stream)
{
    if (x == nullptr || update == nullptr || d > kMaxElements)
        return MARSIT_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(update, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    hipLaunchKernelGGL(apply_update_kernel<kStreamCols>, dim3(stream_blocks((d + 3) >> 2, kStreamCols)), dim3(kSyncBlock), 0,
                       static_cast<hipStream_t>(stream), x, update, d);
    return finish_launch();
}

int marsit_local_momentum(float *buf, const float *grad, float *g_out, uint32_t M, uint64_t d,
                          uint64_t ld, float beta, float eta_l, void *stream)
{
    if (buf == nullptr || grad == nullptr || g_out == nullptr || M == 0 || M > MARSIT_MAX_WORKERS ||
        ld < d || d > kMaxElements || !std::isfinite(beta) || !std::isfinite(eta_l) || buf == grad ||
        buf == g_out)
        return MARSIT_EINVAL;
    if (!aligned_to(buf, 4) || !aligned_to(grad, 4) || !aligned_to(g_out, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    hipLaunchKernelGGL(local_momentum_kernel<kStreamCols>, dim3(stream_blocks((d + 3) >> 2, kStreamCols), M), dim3(kSyncBlock),
                       throttle_lds_bytes(16),
                       static_cast<hipStream_t>(stream), buf, grad, g_out, d, ld, beta, eta_l);
    return finish_launch();
}

int marsit_local_adam(float *mom1, float *mom2, const float *grad, float *g_out, uint32_t M, uint64_t d,
                      uint64_t ld, float beta1, float beta2, float eps, float eta_l, float bias1,
                      float bias2, void *stream)
{
    if (mom1 == nullptr || mom2 == nullptr || grad == nullptr || g_out == nullptr || M == 0 ||
        M > MARSIT_MAX_WORKERS || ld < d || d > kMaxElements || !std::isfinite(beta1) ||
        !std::isfinite(beta2) || !std::isfinite(eps) || !std::isfinite(eta_l) || !std::isfinite(bias1) ||
        !std::isfinite(bias2) || bias1 == 0.0f || bias2 == 0.0f || mom1 == mom2 || mom1 == grad ||
        mom2 == grad || mom1 == g_out || mom2 == g_out)
        return MARSIT_EINVAL;
    if (!aligned_to(mom1, 4) || !aligned_to(mom2, 4) || !aligned_to(grad, 4) || !aligned_to(g_out, 4))
        return MARSIT_EALIGN;
    if (d == 0)
        return MARSIT_OK;
    const float rest1 = 1.0f - beta1;
    const float rest2 = 1.0f - beta2;
    hipLaunchKernelGGL(local_adam_kernel<kStreamCols>, dim3(stream_blocks((d + 3) >> 2, kStreamCols), M),
                       dim3(kSyncBlock), throttle_lds_bytes(16), static_cast<hipStream_t>(stream), mom1, mom2, grad,
                       g_out, d, ld, beta1, rest1, beta2, rest2, eps, eta_l, bias1, bias2);
    return finish_launch();
}

}   // extern "C"
