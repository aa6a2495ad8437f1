// Shared host/device helpers of the LOOKAT HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "lookat.h"

namespace lookat {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kCentroids = 256;  // K fixed by the method: one byte per code

// Records a message for lookat_last_error() and returns `status` (host).
int fail(int status, const char *fmt, ...);
void clear_error();

// Common argument checks of every entry point (host).  Returns LOOKAT_OK or a failure.
int check_shape(const lookat_shape *s);
int check_launch(const char *what);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#if defined(__HIPCC__)

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off);
    return v;
}

// 2^x on the transcendental unit; 2^-inf = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

#endif  // __HIPCC__

}  // namespace lookat
