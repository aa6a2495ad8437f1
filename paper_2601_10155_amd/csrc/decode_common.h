// Device helpers shared by the decode kernels (gfx950 only): tile constants, buffer descriptors, the
// per-key code fetch and lookup-and-sum (paper Sec. 3.5), value-row loads and the online-softmax state.
#pragma once

#include "common.h"

namespace lookat {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWave;
constexpr int kTile = 64;          // keys per wavefront tile: one key per lane in the score phase
constexpr int kXcds = 8;           // accelerator dies; workgroup ids are dealt round-robin to them
constexpr float kLog2e = 1.4426950408889634f;

typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

// Buffer descriptor over [base, base + bytes): loads past the end return zero instead of
// faulting, which is how ragged tiles and the prefetch past the last tile are handled.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// The m codes of one key, fetched with a single load when m is 2, 4, 8 or 16.
template <int M>
struct KeyCodes {
    static constexpr int kWords = (M + 3) / 4;
    uint32_t w[kWords];
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rc, uint32_t byte_off)
    {
        if constexpr (M == 2) {
            w[0] = __builtin_amdgcn_raw_buffer_load_b16(rc, byte_off, 0, 0);
        } else if constexpr (M == 4) {
            w[0] = __builtin_amdgcn_raw_buffer_load_b32(rc, byte_off, 0, 0);
        } else if constexpr (M == 8) {
            const v2u t = __builtin_amdgcn_raw_buffer_load_b64(rc, byte_off, 0, 0);
            w[0] = t.x;
            w[1] = t.y;
        } else {
            static_assert(M == 16, "vector code loads exist for m = 2, 4, 8, 16");
            const v4u t = __builtin_amdgcn_raw_buffer_load_b128(rc, byte_off, 0, 0);
            w[0] = t.x;
            w[1] = t.y;
            w[2] = t.z;
            w[3] = t.w;
        }
    }
    // Unscaled ADC score: sum_i LUT_i[code_i], i ascending.
    __device__ __forceinline__ float score(const float *lut_s) const
    {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < M; ++i) {
            const uint32_t byte = (w[i / 4] >> (8 * (i % 4))) & 0xffu;
            s += lut_s[i * kCentroids + byte];
        }
        return s;
    }
};

// Runtime m: byte loads (used for m = 1 and m = 32 and any m without a vector load).
__device__ __forceinline__ float score_bytes(const float *lut_s, __amdgpu_buffer_rsrc_t rc, uint32_t byte_off, int m)
{
    float s = 0.f;
    for (int i = 0; i < m; ++i)
        s += lut_s[i * kCentroids + __builtin_amdgcn_raw_buffer_load_b8(rc, byte_off + i, 0, 0)];
    return s;
}

__device__ __forceinline__ void fma_row(float (&acc)[8], float p, const v4u &v)
{
    const __half2 *h = reinterpret_cast<const __half2 *>(&v);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float2 f = __half22float2(h[k]);
        acc[2 * k] = fmaf(p, f.x, acc[2 * k]);
        acc[2 * k + 1] = fmaf(p, f.y, acc[2 * k + 1]);
    }
}

// acc += p_j * row_j for the CH row groups c0 .. c0+CH-1 held in v; p_j is the weight held by
// lane c0+j of the caller's LPR-lane group.
template <int LPR, int CH, int J = 0>
__device__ __forceinline__ void fma_rows(float (&acc)[8], float p, const v4u (&v)[CH], int c0)
{
    if constexpr (J < CH) {
        // c0 is 0 or 8 (CH = 8 whenever a tile has more than one chunk)
        float pj;
        if constexpr (LPR <= 8) {
            pj = group_broadcast<LPR, J>(p);
        } else {
            pj = (c0 == 0) ? group_broadcast<LPR, J>(p)
               : (c0 == 8) ? group_broadcast<LPR, (J + 8) % LPR>(p)
               : (c0 == 16) ? group_broadcast<LPR, (J + 16) % LPR>(p)
                            : group_broadcast<LPR, (J + 24) % LPR>(p);
        }
        fma_row(acc, pj, v[J]);
        fma_rows<LPR, CH, J + 1>(acc, p, v, c0);
    }
}

// Loads CH consecutive wave-wide row groups of the tile starting at key kb, from group g0.
template <int DK, int CH>
__device__ __forceinline__ void load_rows(v4u (&v)[CH], __amdgpu_buffer_rsrc_t rv, uint32_t kb, int g0, int lane)
{
    // lane (rowin, sub) reads 16 bytes at row*DK*2 + sub*16 = (row0*DK*2) + lane*16: 1 KB per load
    constexpr uint32_t kGroupBytes = kWave * 16;
    // Non-temporal (aux bit 1): the rows are read once and should not displace tables, codebooks and
    // queries from the caches; measured 11.94 -> 11.29 us per fused launch at batch 32 x 12 heads x 1024
    // keys (the same hint on the code loads as well: 11.39).
    constexpr int kStreamOnce = 2;
#pragma unroll
    for (int j = 0; j < CH; ++j)
        v[j] = __builtin_amdgcn_raw_buffer_load_b128(rv, kb * (DK * 2) + (g0 + j) * kGroupBytes + lane * 16, 0,
                                                     kStreamOnce);
}

// Online-softmax state of one wavefront (base-2 exponent domain), for each of the G query heads
// that share the key/value head (G = 1: plain multi-head attention).
template <int G>
struct SoftmaxState {
    float m_run[G];    // running max of scale*log2e*s over the keys seen so far
    float z[G];        // this lane's share of the running sum of weights
    float acc[G][8];   // this lane's slice of sum_l w_l v_l
    __device__ __forceinline__ SoftmaxState()
    {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            m_run[g] = -INFINITY;
            z[g] = 0.f;
#pragma unroll
            for (int d = 0; d < 8; ++d)
                acc[g][d] = 0.f;
        }
    }
};

}  // namespace lookat
