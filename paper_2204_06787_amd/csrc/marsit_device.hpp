// Device-side building blocks of the Marsit one-bit pass for gfx950 (64-lane wavefronts).
//
// Lane layout used by every kernel that touches fp32 vectors with 128-bit accesses: a lane owns a
// "column" of 4 consecutive elements e = 4*col .. 4*col+3.  Sixteen consecutive lanes (one DPP row)
// own one packed 64-bit sign word w = col / 16, and lane q = col % 16 of that row owns bits
// 4q .. 4q+3 of it.  One Philox4x32-10 call yields four 32-bit words, so counter word 0 = q gives
// a lane exactly the four draws of its four bits: draw j of packed word w is output j % 4 of
// block j / 4.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace marsit {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Philox4x32-10 constants (Salmon, Moraes, Dror, Shaw, SC'11): the two multipliers and the two
// Weyl increments of the key schedule.
constexpr uint32_t kPhiloxMulA = 0xD2511F53u;
constexpr uint32_t kPhiloxMulB = 0xCD9E8D57u;
constexpr uint32_t kPhiloxWeylA = 0x9E3779B9u;
constexpr uint32_t kPhiloxWeylB = 0xBB67AE85u;

// a ^ b ^ c.  On the device one three-input bitwise instruction (v_bitop3_b32, truth table 0x96),
// which the compiler does not form by itself from two XORs: a Philox call is then 20 multiply-adds
// and 20 of these instead of 20 + 40 (the kernels that only draw run 1.2 x faster; the memory-bound
// ones do not change).  The host version serves marsit_philox4x32_10.
__host__ __device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
#else
    return a ^ b ^ c;
#endif
}

__host__ __device__ __forceinline__ void philox_round(uint32_t &c0, uint32_t &c1, uint32_t &c2,
                                                      uint32_t &c3, uint32_t k0, uint32_t k1)
{
    const uint64_t pa = static_cast<uint64_t>(kPhiloxMulA) * c0;
    const uint64_t pb = static_cast<uint64_t>(kPhiloxMulB) * c2;
    const uint32_t n0 = xor3(static_cast<uint32_t>(pb >> 32), c1, k0);
    const uint32_t n2 = xor3(static_cast<uint32_t>(pa >> 32), c3, k1);
    c1 = static_cast<uint32_t>(pb);
    c3 = static_cast<uint32_t>(pa);
    c0 = n0;
    c2 = n2;
}

// Ten rounds; the key advances by the Weyl constants between rounds.
__host__ __device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2,
                                                       uint32_t c3, uint32_t k0, uint32_t k1,
                                                       uint32_t out[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        philox_round(c0, c1, c2, c3, k0 + static_cast<uint32_t>(r) * kPhiloxWeylA,
                     k1 + static_cast<uint32_t>(r) * kPhiloxWeylB);
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

// floor(2^32 / fold) for fold >= 2: a 32-bit draw below it has probability 1/fold (Eq. 2).
__host__ __device__ constexpr uint32_t keep_threshold(uint32_t fold)
{
    return static_cast<uint32_t>((static_cast<uint64_t>(1) << 32) / fold);
}

// hop ids of the torus schedule: row phase carries the row, column phase is flagged in bit 16.
__host__ __device__ constexpr uint32_t row_hop_id(uint32_t row, uint32_t hop) { return (row << 8) | hop; }
__host__ __device__ constexpr uint32_t col_hop_id(uint32_t hop) { return (1u << 16) | hop; }

// Reduction tree: hop id of the merge at `level` whose receiver is worker `receiver`.
__host__ __device__ constexpr uint32_t tree_hop_id(uint32_t level, uint32_t receiver)
{
    return (2u << 16) | (level << 8) | receiver;
}

// Keep-local threshold when the received vector stands for w_recv workers and the local one for
// w_local (Eq. 2 with the local share in place of 1/m): floor(2^32 * w_local / (w_recv + w_local)).
// w_recv must be >= 1 (w_recv = 0 means "always local" and is handled by the callers).
__host__ __device__ constexpr uint32_t weighted_threshold(uint32_t w_recv, uint32_t w_local)
{
    return static_cast<uint32_t>((static_cast<uint64_t>(w_local) << 32) /
                                 (static_cast<uint64_t>(w_recv) + w_local));
}

__device__ __forceinline__ uint32_t f32_bits(float x) { return __float_as_uint(x); }

// ---- 128-bit / guarded accesses ---------------------------------------------------------------

// 128-bit accesses are made through a vector type that promises dword alignment only: gfx950
// global memory instructions take any dword-aligned address for a four-dword access, so rows that
// do not start on a 16-byte boundary (odd row strides, offset bases) use the same instructions.
typedef f32x4 f32x4_dw __attribute__((aligned(4)));

// Four consecutive floats at p.  `vec`: all four are inside the vector (p is 4-byte aligned, as
// every fp32 pointer of the library must be).  Otherwise the first n_valid (0..4) are read one by
// one, the rest are +0.  STREAMING marks data that is read once (non-temporal hint).
template <bool STREAMING = true>
__device__ __forceinline__ f32x4 load4(const float *p, bool vec, uint32_t n_valid)
{
    if (vec) {
        if (STREAMING)
            return __builtin_nontemporal_load(reinterpret_cast<const f32x4_dw *>(p));
        return *reinterpret_cast<const f32x4_dw *>(p);
    }
    f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (n_valid > 0) v.x = p[0];
    if (n_valid > 1) v.y = p[1];
    if (n_valid > 2) v.z = p[2];
    if (n_valid > 3) v.w = p[3];
    return v;
}

template <bool STREAMING>
__device__ __forceinline__ void store4(float *p, f32x4 v, bool vec, uint32_t n_valid)
{
    if (vec) {
        if (STREAMING)
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4_dw *>(p));
        else
            *reinterpret_cast<f32x4_dw *>(p) = v;
        return;
    }
    if (n_valid > 0) p[0] = v.x;
    if (n_valid > 1) p[1] = v.y;
    if (n_valid > 2) p[2] = v.z;
    if (n_valid > 3) p[3] = v.w;
}

// Streaming (read-once / write-once) 128-bit accesses of whole columns: the non-temporal hint keeps
// the lines from displacing each other in L2 and the memory-side cache; with 2M+ concurrent
// streams it is worth about 10 % of bandwidth on MI355X.
__device__ __forceinline__ f32x4 load4_stream(const float *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4_dw *>(p));
}

__device__ __forceinline__ void store4_stream(float *p, f32x4 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4_dw *>(p));
}

// ---- DPP: OR over the 8 lanes of a half row ------------------------------------------------------

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t x)
{
    return static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, 0xF, 0xF, false));
}

// Every lane must be active when this is called.  Afterwards each lane holds the OR of the
// values of the 8 lanes of its half row (lanes 8k .. 8k+7 of the wavefront).
__device__ __forceinline__ uint32_t half_row_or(uint32_t x)
{
    x |= dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]: neighbour at distance 1
    x |= dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]: neighbour at distance 2
    x |= dpp_move<0x141>(x);   // row_half_mirror: lane i <-> 7-i, the other quad of the half row
    return x;
}

// Lane q (0..15 of its row) contributes nibble `nib` = bits 4q..4q+3 of its row's 64-bit word.
// Returns, in every lane, the 32-bit half of that word the lane belongs to (q < 8: low half).
__device__ __forceinline__ uint32_t gather_half_word(uint32_t nib, uint32_t q)
{
    return half_row_or(nib << ((q & 7u) * 4u));
}

}   // namespace marsit
