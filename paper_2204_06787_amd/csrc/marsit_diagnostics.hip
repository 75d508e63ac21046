// Diagnostics of Section 3.2.2 / Fig. 2(b) and the strawman they are measured against: sign of
// the non-compressed aggregate, majority vote, matching count, SSDM stochastic sign and cascading
// compression.

#include "marsit_device.hpp"
#include "marsit_host.hpp"

namespace marsit {

// -------------------------------------------------------------------------------------------------
// Diagnostics of Section 3.2.2 / Fig. 2(b): sign of the non-compressed aggregate, majority vote,
// and the number of positions at which two sign bitmaps agree (numerator of the matching rate).
// -------------------------------------------------------------------------------------------------
enum VoteMode { kAggregateSign = 0, kMajorityVote = 1 };

template <int MODE>
__global__ void __launch_bounds__(kBlock)
vote_kernel(const float *__restrict__ g, const float *__restrict__ c, uint32_t *__restrict__ bits32,
            uint32_t M, uint64_t d, uint64_t ld)
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
        const bool vec = full;
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
                            const float *c, uint64_t n, double *partial)
{
    __shared__ double wave_sum[kBlock / 64];
    const uint64_t n_cols = (n + 3) >> 2;
    double acc = 0.0;
    for (uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x; col < n_cols;
         col += static_cast<uint64_t>(gridDim.x) * kBlock) {
        const uint64_t e = col << 2;
        const bool full = e + 4 <= n;
        const uint32_t n_valid = full ? 4u : static_cast<uint32_t>(n - e);
        const f32x4 t = cascade_value(recv32, recv_norm, g, c, col, full, n_valid);
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
                    uint32_t hop_id, uint32_t key0, uint32_t key1)
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
        const f32x4 t = cascade_value(recv32, recv_norm, g, c, col, full, n_valid);
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
    // lane = one column of 4 elements (nibble col % 8 of 32-bit half col / 8)
    const uint64_t col = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    const uint64_t e = col << 2;
    if (e >= n)
        return;
    const float norm = *norm_ptr;
    const uint32_t nib = (bits32[col >> 3] >> ((static_cast<uint32_t>(col) & 7u) * 4u)) & 0xFu;
    const uint32_t n_valid = (e + 4 <= n) ? 4u : static_cast<uint32_t>(n - e);
    for (uint32_t j = 0; j < n_valid; ++j)
        update[e + j] = (((nib >> j) & 1u) ? norm : -norm) / workers;
}

}   // namespace marsit

using namespace marsit;

extern "C" {

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
    const dim3 grid(blocks_for((d + 3) >> 2)), block(kBlock);
    uint32_t *bits32 = reinterpret_cast<uint32_t *>(bits_out);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mode == kAggregateSign)
        hipLaunchKernelGGL(vote_kernel<kAggregateSign>, grid, block, 0, s, g, c, bits32, M, d, ld);
    else
        hipLaunchKernelGGL(vote_kernel<kMajorityVote>, grid, block, 0, s, g, c, bits32, M, d, ld);
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
    const uint64_t n_cols = (n + 3) >> 2;
    uint32_t n_partials = blocks_for(n_cols);
    if (n_partials > kCascadeMaxPartials)
        n_partials = kCascadeMaxPartials;
    double *partial = static_cast<double *>(workspace);
    const uint32_t *recv32 = reinterpret_cast<const uint32_t *>(recv_bits);
    hipLaunchKernelGGL(cascade_norm_partial_kernel, dim3(n_partials), dim3(kBlock), 0, s, recv32,
                       recv_norm, g, c, n, partial);
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
                       static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
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
        hipLaunchKernelGGL(cascade_decode_kernel, dim3(blocks_for((n + 3) >> 2)), dim3(kBlock), 0, s,
                           reinterpret_cast<const uint32_t *>(bits), norms_out + i, update_out + e0, n,
                           static_cast<float>(M));
        const int rc = finish_launch();
        if (rc != MARSIT_OK)
            return rc;
    }
    return MARSIT_OK;
}

}   // extern "C"
