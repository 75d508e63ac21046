// Host-side helpers shared by the translation units of libmarsit (internal, not installed).
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>

#include "marsit.h"

#ifndef MARSIT_STREAMING_STORES
#define MARSIT_STREAMING_STORES 1
#endif

namespace marsit {

constexpr int kBlock = 256;       // every kernel but the fused ones
constexpr int kSyncBlock = 64;    // fused kernels: one wavefront per workgroup
// Largest vector any entry point takes.  The widest launches use one work-item per column of 4
// elements, rounded up to whole workgroups of kBlock, and a launch may not reach 2^32 work-items
// in x: ceil(d / 4) rounded up to 256 stays below 2^32 exactly when d <= 2^34 - 1024.
constexpr uint64_t kMaxElements = MARSIT_MAX_ELEMENTS;
static_assert(((kMaxElements + 3) / 4 + 255) / 256 * 256 < (static_cast<uint64_t>(1) << 32),
              "a launch over MARSIT_MAX_ELEMENTS elements must stay below 2^32 work-items");
static_assert((((kMaxElements + 1) + 3) / 4 + 255) / 256 * 256 >= (static_cast<uint64_t>(1) << 32),
              "MARSIT_MAX_ELEMENTS is the largest size one launch covers");

// hipError_t of the last failed HIP call of this thread (marsit_last_hip_error)
extern thread_local int tls_last_hip_error;

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

// Dynamic LDS bytes per workgroup that leave room for exactly `waves` one-wavefront workgroups on
// a CU: the kernels never touch it, it only limits how many of them are resident.
inline uint32_t throttle_lds_bytes(uint32_t waves)
{
    constexpr uint32_t lds_per_cu = 160u * 1024u;   // gfx950; the runtime attribute reports 64 KB
    // a few per cent below an even share: with an exact share one workgroup fewer fits.  (gfx950
    // takes dynamic requests up to the whole 160 KB; two workgroups per CU ask for 77.5 KB.)
    return ((lds_per_cu / waves) * 31u / 32u) & ~511u;
}

// Fine part bounds of the schedule (see marsit_split_bounds in marsit.h).
int split_bounds_host(uint64_t n_words, uint32_t M, uint32_t grid_x, uint64_t *bounds);

}   // namespace marsit
