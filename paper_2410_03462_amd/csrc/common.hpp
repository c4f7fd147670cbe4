// Internal helpers shared by the translation units of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "grf.h"

namespace grf {

constexpr int kWave = 64;                 // CDNA wavefront width
constexpr size_t kAlign = 256;            // alignment of every workspace section

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Thread-local error message behind grf_last_error().
char* error_buffer();
grf_status fail(grf_status code, const char* fmt, ...);

#define GRF_HIP_TRY(expr)                                                                      \
    do {                                                                                       \
        hipError_t err__ = (expr);                                                             \
        if (err__ != hipSuccess)                                                               \
            return ::grf::fail(GRF_EHIP, "%s failed: %s", #expr, hipGetErrorString(err__));    \
    } while (0)

#define GRF_LAUNCH_CHECK(name)                                                                 \
    do {                                                                                       \
        hipError_t err__ = hipGetLastError();                                                  \
        if (err__ != hipSuccess)                                                               \
            return ::grf::fail(GRF_EHIP, "launch of %s failed: %s", name, hipGetErrorString(err__)); \
    } while (0)

// Exclusive prefix sum in place over counts[0..n-1]; counts[n] receives the total (clamped to
// INT32_MAX) and *total64 the unclamped total.  Enqueued on `stream`.
grf_status exclusive_scan_inplace(int32_t* counts, int64_t n, long long* total64, hipStream_t stream);

// data[0..n-1] = value.
grf_status fill_i32(int32_t* data, int64_t n, int32_t value, hipStream_t stream);

// ---- wave-level device helpers ------------------------------------------------------------

__device__ __forceinline__ int lane_id() { return static_cast<int>(threadIdx.x) & (kWave - 1); }

// Number of set bits of `mask` strictly below this lane.
__device__ __forceinline__ int prefix_popcount(unsigned long long mask)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask), 0u));
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

}  // namespace grf
