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

// ---- cross-lane moves on the vector ALU (DPP / lane swaps): no LDS traffic -----------
// dpp_mov<CTRL>(x): lane i receives x from the lane the DPP control selects.
//   quad_perm [a,b,c,d] = a | b<<2 | c<<4 | d<<6;  row_shl:n = 0x100+n;  row_shr:n = 0x110+n;
//   row_ror:n = 0x120+n;  row_mirror = 0x140;  row_half_mirror = 0x141;  row_newbcast:n = 0x150+n
//   (a row = 16 lanes)
template <int CTRL, int BANK_MASK = 0xf>
__device__ __forceinline__ float dpp_mov(float keep, float x)
{
    return __int_as_float(
        __builtin_amdgcn_update_dpp(__float_as_int(keep), __float_as_int(x), CTRL, 0xf, BANK_MASK, false));
}

// x[lane] and x[lane ^ 16] (swap of odd/even 16-lane rows), x[lane ^ 32] (swap of halves)
__device__ __forceinline__ void lanes_xor16(float x, float &a, float &b)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}
__device__ __forceinline__ void lanes_xor32(float x, float &a, float &b)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}

// All-lanes reductions over the 64-lane wavefront; every lane ends with the result.
__device__ __forceinline__ float wave_max(float v)
{
    float a, b;
    v = fmaxf(v, dpp_mov<0xB1>(v, v));    // quad_perm [1,0,3,2]: lane ^ 1
    v = fmaxf(v, dpp_mov<0x4E>(v, v));    // quad_perm [2,3,0,1]: lane ^ 2
    v = fmaxf(v, dpp_mov<0x141>(v, v));   // row_half_mirror: the other quad of each 8
    v = fmaxf(v, dpp_mov<0x140>(v, v));   // row_mirror: the other 8 of each 16
    lanes_xor16(v, a, b);
    v = fmaxf(a, b);
    lanes_xor32(v, a, b);
    return fmaxf(a, b);
}

__device__ __forceinline__ float wave_sum(float v)
{
    float a, b;
    v += dpp_mov<0xB1>(v, v);
    v += dpp_mov<0x4E>(v, v);
    v += dpp_mov<0x141>(v, v);
    v += dpp_mov<0x140>(v, v);
    lanes_xor16(v, a, b);
    v = a + b;
    lanes_xor32(v, a, b);
    return a + b;
}

// Sum over the lanes that share (lane % G), G a power of two in [4, 32]: every lane ends
// with the sum of its residue class.
template <int G>
__device__ __forceinline__ float sum_over_lane_classes(float v)
{
    float a, b;
    if constexpr (G <= 4)
        v += dpp_mov<0x124>(v, v);        // row_ror:4
    if constexpr (G <= 8)
        v += dpp_mov<0x128>(v, v);        // row_ror:8
    if constexpr (G <= 16) {
        lanes_xor16(v, a, b);
        v = a + b;
    }
    lanes_xor32(v, a, b);
    return a + b;
}

// Value of lane J of the caller's aligned group of G consecutive lanes.
template <int G, int J>
__device__ __forceinline__ float group_broadcast(float x)
{
    if constexpr (G == 4) {
        return dpp_mov<J | (J << 2) | (J << 4) | (J << 6)>(x, x);
    } else if constexpr (G == 8) {
        constexpr int Q = J & 3;
        const float t = dpp_mov<Q | (Q << 2) | (Q << 4) | (Q << 6)>(x, x);   // lane Q of every quad
        if constexpr (J < 4)
            return dpp_mov<0x114, 0xA>(t, t);   // row_shr:4 into quads 1 and 3
        else
            return dpp_mov<0x104, 0x5>(t, t);   // row_shl:4 into quads 0 and 2
    } else if constexpr (G == 16) {
        return dpp_mov<0x150 + J>(x, x);        // row_newbcast:J -- lane J of the 16-lane row to all its lanes
    } else {
        return __shfl(x, (int)((threadIdx.x & (kWave - 1) & ~(G - 1)) + J));
    }
}

// Argmin over the 256 centroids with the encoder's rule (strict '<' scan over ascending index).
// Distances are mapped to an order value: the distance itself; a NaN becomes +inf (it never
// wins), except at centroid 0, where it becomes -1 (the scan starts there and nothing compares
// below a NaN).  The smallest order value with the lowest index is then exactly the scan's result.
__device__ __forceinline__ double argmin_value(double d, int c)
{
    return (d != d) ? (c == 0 ? -1.0 : (double)INFINITY) : d;
}
template <int CTRL>
__device__ __forceinline__ double dmin_dpp(double x)
{
    const uint64_t u = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)u, (int)(uint32_t)u, CTRL, 0xf, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(u >> 32), (int)(uint32_t)(u >> 32), CTRL,
                                                               0xf, 0xf, false);
    return fmin(x, __longlong_as_double((long long)(((uint64_t)hi << 32) | lo)));
}
// N independent minima over the wavefront, reduced in lock step (the chains interleave);
// every lane ends with all N results.
template <int N>
__device__ __forceinline__ void dmin_wave(double (&x)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i)
        x[i] = dmin_dpp<0xB1>(x[i]);    // lane ^ 1
#pragma unroll
    for (int i = 0; i < N; ++i)
        x[i] = dmin_dpp<0x4E>(x[i]);    // lane ^ 2
#pragma unroll
    for (int i = 0; i < N; ++i)
        x[i] = dmin_dpp<0x141>(x[i]);   // other quad of each 8
#pragma unroll
    for (int i = 0; i < N; ++i)
        x[i] = dmin_dpp<0x140>(x[i]);   // other 8 of each 16
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const uint64_t u = (uint64_t)__double_as_longlong(x[i]);
        const auto l = __builtin_amdgcn_permlane16_swap((uint32_t)u, (uint32_t)u, false, false);
        const auto h = __builtin_amdgcn_permlane16_swap((uint32_t)(u >> 32), (uint32_t)(u >> 32), false, false);
        x[i] = fmin(__longlong_as_double((long long)(((uint64_t)h[0] << 32) | l[0])),
                    __longlong_as_double((long long)(((uint64_t)h[1] << 32) | l[1])));
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const uint64_t u = (uint64_t)__double_as_longlong(x[i]);
        const auto l = __builtin_amdgcn_permlane32_swap((uint32_t)u, (uint32_t)u, false, false);
        const auto h = __builtin_amdgcn_permlane32_swap((uint32_t)(u >> 32), (uint32_t)(u >> 32), false, false);
        x[i] = fmin(__longlong_as_double((long long)(((uint64_t)h[0] << 32) | l[0])),
                    __longlong_as_double((long long)(((uint64_t)h[1] << 32) | l[1])));
    }
}

// 2^x on the transcendental unit; 2^-inf = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

#endif  // __HIPCC__

}  // namespace lookat
