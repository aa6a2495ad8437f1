// Key encoding (paper Sec. 3.4, "Encoding"): per key and subspace, the index of the
// nearest centroid.  The distance is evaluated in fp64 with one rounding per subtract,
// multiply and add, coordinates ascending, and a strict '<' scan over ascending
// centroid index, so the code is unique and identical on every IEEE machine.
//
// This translation unit must be compiled with -ffp-contract=off: a fused multiply-add
// in the distance would change near-tie decisions.
#include <cstdlib>

#include "common.h"

#pragma clang fp contract(off)

namespace lookat {

constexpr int kEncThreads = 256;
constexpr int kEncLdsDoubles = 4096;  // centroid chunk staged in LDS: 32 KB of fp64

template <typename T>
__device__ __forceinline__ double widen(T v);
template <>
__device__ __forceinline__ double widen<float>(float v) { return (double)v; }
template <>
__device__ __forceinline__ double widen<__half>(__half v) { return (double)__half2float(v); }

// One block = 256 keys of one head, one subspace.  The key sub-vector lives in
// registers as fp64; the centroids of the subspace are staged in LDS as fp64 and read
// by all lanes at the same address (LDS broadcast, conflict free).
//   grid = (ceil(B*N / 256), m, H)
template <typename KT, int DSUB>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(const KT *__restrict__ keys,
                                                             const float *__restrict__ codebooks,
                                                             uint8_t *__restrict__ codes, int64_t code_stride_bh,
                                                             int B, int H, int64_t N, int d_k, int m)
{
    __shared__ double cb_s[kEncLdsDoubles];
    constexpr int KC = (kEncLdsDoubles / DSUB) < kCentroids ? (kEncLdsDoubles / DSUB) : kCentroids;

    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int64_t r = (int64_t)blockIdx.x * kEncThreads + threadIdx.x;  // flat (b, n)
    const bool live = r < (int64_t)B * N;
    const int64_t b = live ? r / N : 0;
    const int64_t n = live ? r % N : 0;
    const int64_t bh = b * H + h;

    double x[DSUB];
    {
        const KT *src = keys + (bh * N + n) * d_k + (int64_t)i * DSUB;
#pragma unroll
        for (int j = 0; j < DSUB; ++j)
            x[j] = live ? widen<KT>(src[j]) : 0.0;
    }

    const float *cb = codebooks + ((int64_t)h * m + i) * kCentroids * DSUB;
    double best = 0.0;
    int best_c = 0;
    for (int c0 = 0; c0 < kCentroids; c0 += KC) {
        __syncthreads();
        for (int e = threadIdx.x; e < KC * DSUB; e += kEncThreads)
            cb_s[e] = (double)cb[(int64_t)c0 * DSUB + e];
        __syncthreads();
        for (int c = 0; c < KC; ++c) {
            const double *y = cb_s + c * DSUB;
            double acc = 0.0;
#pragma unroll
            for (int j = 0; j < DSUB; ++j) {
                double diff = x[j] - y[j];
                double sq = diff * diff;
                acc = acc + sq;
            }
            // first centroid initialises the scan; afterwards strict '<' keeps the lowest index
            if ((c0 + c) == 0 || acc < best) {
                best = acc;
                best_c = c0 + c;
            }
        }
    }
    if (live)
        codes[bh * code_stride_bh + n * m + i] = (uint8_t)best_c;
}

// Any d_sub: the key sub-vector is re-read from memory per centroid (slow, small shapes only).
template <typename KT>
__global__ __launch_bounds__(kEncThreads) void encode_generic_kernel(const KT *__restrict__ keys,
                                                                     const float *__restrict__ codebooks,
                                                                     uint8_t *__restrict__ codes,
                                                                     int64_t code_stride_bh, int B, int H, int64_t N,
                                                                     int d_k, int m)
{
    const int d_sub = d_k / m;
    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int64_t r = (int64_t)blockIdx.x * kEncThreads + threadIdx.x;
    if (r >= (int64_t)B * N)
        return;
    const int64_t b = r / N, n = r % N;
    const int64_t bh = b * H + h;
    const KT *src = keys + (bh * N + n) * d_k + (int64_t)i * d_sub;
    const float *cb = codebooks + ((int64_t)h * m + i) * kCentroids * d_sub;
    double best = 0.0;
    int best_c = 0;
    for (int c = 0; c < kCentroids; ++c) {
        double acc = 0.0;
        for (int j = 0; j < d_sub; ++j) {
            double diff = widen<KT>(src[j]) - (double)cb[(int64_t)c * d_sub + j];
            double sq = diff * diff;
            acc = acc + sq;
        }
        if (c == 0 || acc < best) {
            best = acc;
            best_c = c;
        }
    }
    codes[bh * code_stride_bh + n * m + i] = (uint8_t)best_c;
}

// ---- few keys per head (decode-time append) -------------------------------------------
// With a handful of keys per head the thread-per-key kernel above leaves the chip empty and
// each thread walks all 256 centroids serially.  Here the centroids are spread over the
// threads instead: one block = one (head, subspace) and up to kEncFewKeys keys; thread c
// holds centroid c in registers as fp64, evaluates its distance to every key of the block
// (same arithmetic, same order) and the block takes the argmin over (distance, index).
constexpr int kEncFewKeys = 8;

template <typename KT, int DSUB>
__global__ __launch_bounds__(kCentroids) void encode_few_kernel(const KT *__restrict__ keys,
                                                                const float *__restrict__ codebooks,
                                                                uint8_t *__restrict__ codes, int64_t code_stride_bh,
                                                                int B, int H, int64_t N, int d_k, int m)
{
    __shared__ double x_s[kEncFewKeys][DSUB];
    __shared__ double red_d[kEncFewKeys][kCentroids / kWave];
    __shared__ int red_c[kEncFewKeys][kCentroids / kWave];

    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int c = threadIdx.x;
    const int lane = c & (kWave - 1), wave = c / kWave;
    const int64_t r0 = (int64_t)blockIdx.x * kEncFewKeys;   // first flat (b, n) of the block
    const int64_t rows = (int64_t)B * N;

    for (int e = threadIdx.x; e < kEncFewKeys * DSUB; e += kCentroids) {
        const int64_t r = r0 + e / DSUB;
        double v = 0.0;
        if (r < rows) {
            const int64_t b = r / N, n = r % N;
            v = widen<KT>(keys[((b * H + h) * N + n) * d_k + (int64_t)i * DSUB + e % DSUB]);
        }
        x_s[e / DSUB][e % DSUB] = v;
    }
    double y[DSUB];
    {
        const float *src = codebooks + (((int64_t)h * m + i) * kCentroids + c) * DSUB;
#pragma unroll
        for (int j = 0; j < DSUB; ++j)
            y[j] = (double)src[j];
    }
    __syncthreads();

    // Distances of centroid c to the block's keys, then per key the minimum over the wavefront's 64
    // centroids (cross-lane moves on the vector ALU, the eight chains interleaved) and the lowest
    // lane that holds it: the serial scan's choice among exact ties.
    double dv[kEncFewKeys], dm[kEncFewKeys];
#pragma unroll
    for (int k = 0; k < kEncFewKeys; ++k) {
        double acc = 0.0;
#pragma unroll
        for (int j = 0; j < DSUB; ++j) {
            double diff = x_s[k][j] - y[j];
            double sq = diff * diff;
            acc = acc + sq;
        }
        dv[k] = argmin_value(acc, c);
        dm[k] = dv[k];
    }
    dmin_wave<kEncFewKeys>(dm);
#pragma unroll
    for (int k = 0; k < kEncFewKeys; ++k) {
        const uint64_t holders = __ballot(dv[k] == dm[k]);
        if (lane == 0) {
            red_d[k][wave] = dm[k];
            red_c[k][wave] = wave * kWave + (int)__builtin_ctzll(holders);
        }
    }
    __syncthreads();
    if (threadIdx.x < kEncFewKeys) {
        const int k = threadIdx.x;
        const int64_t r = r0 + k;
        if (r < rows) {
            // wavefronts hold ascending centroid ranges: strict '<' keeps the lowest index on ties
            double bd = red_d[k][0];
            int best = red_c[k][0];
#pragma unroll
            for (int w = 1; w < kCentroids / kWave; ++w) {
                const double d = red_d[k][w];
                const int cw = red_c[k][w];
                const bool better = d < bd;
                bd = better ? d : bd;
                best = better ? cw : best;
            }
            const int64_t b = r / N, n = r % N;
            codes[(b * H + h) * code_stride_bh + n * m + i] = (uint8_t)best;
        }
    }
}

template <typename KT>
static bool launch_encode_few(const lookat_shape *s, int64_t N, const void *keys, const float *codebooks,
                              uint8_t *codes, int64_t code_stride_bh, hipStream_t st)
{
    const int d_sub = s->d_k / s->m;
    const int64_t rows = (int64_t)s->B * N;
    dim3 grid((unsigned)((rows + kEncFewKeys - 1) / kEncFewKeys), (unsigned)s->m, (unsigned)s->H);
    dim3 block(kCentroids);
    const KT *k = static_cast<const KT *>(keys);
#define LOOKAT_ENCF_CASE(D)                                                                                     \
    case D:                                                                                                     \
        hipLaunchKernelGGL((encode_few_kernel<KT, D>), grid, block, 0, st, k, codebooks, codes, code_stride_bh, \
                           s->B, s->H, N, s->d_k, s->m);                                                        \
        return true;
    switch (d_sub) {
        LOOKAT_ENCF_CASE(1)
        LOOKAT_ENCF_CASE(2)
        LOOKAT_ENCF_CASE(4)
        LOOKAT_ENCF_CASE(8)
        LOOKAT_ENCF_CASE(16)
        LOOKAT_ENCF_CASE(32)
    default:
        return false;   // no centroid-parallel variant for this sub-vector length
    }
#undef LOOKAT_ENCF_CASE
}

template <typename KT>
static void launch_encode(const lookat_shape *s, int64_t N, const void *keys, const float *codebooks, uint8_t *codes,
                          int64_t code_stride_bh, hipStream_t st)
{
    const int d_sub = s->d_k / s->m;
    const int64_t rows = (int64_t)s->B * N;
    dim3 grid((unsigned)((rows + kEncThreads - 1) / kEncThreads), (unsigned)s->m, (unsigned)s->H);
    dim3 block(kEncThreads);
    const KT *k = static_cast<const KT *>(keys);
#define LOOKAT_ENC_CASE(D)                                                                                      \
    case D:                                                                                                     \
        hipLaunchKernelGGL((encode_kernel<KT, D>), grid, block, 0, st, k, codebooks, codes, code_stride_bh,     \
                           s->B, s->H, N, s->d_k, s->m);                                                        \
        break;
    switch (d_sub) {
        LOOKAT_ENC_CASE(1)
        LOOKAT_ENC_CASE(2)
        LOOKAT_ENC_CASE(4)
        LOOKAT_ENC_CASE(8)
        LOOKAT_ENC_CASE(16)
        LOOKAT_ENC_CASE(32)
        LOOKAT_ENC_CASE(64)
    default:
        hipLaunchKernelGGL((encode_generic_kernel<KT>), grid, block, 0, st, k, codebooks, codes, code_stride_bh,
                           s->B, s->H, N, s->d_k, s->m);
        break;
    }
#undef LOOKAT_ENC_CASE
}

// encode_filter.hip: matrix-core filter in front of the exact rule (d_sub in {4, 8, 16, 32})
bool launch_encode_filter(const lookat_shape *s, int64_t N, const void *keys, int key_dtype, const float *codebooks,
                          uint8_t *codes, int64_t code_stride_bh, hipStream_t st);

}  // namespace lookat

extern "C" int lookat_encode_keys(const lookat_shape *shape, int64_t N, const void *keys, lookat_dtype key_dtype,
                                  const float *codebooks, uint8_t *codes, int64_t code_stride_bh, void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (N < 0)
        return fail(LOOKAT_ERR_SHAPE, "N=%lld is negative", (long long)N);
    if (key_dtype != LOOKAT_F16 && key_dtype != LOOKAT_F32)
        return fail(LOOKAT_ERR_DTYPE, "key_dtype=%d is neither LOOKAT_F16 nor LOOKAT_F32", key_dtype);
    if (N == 0)
        return LOOKAT_OK;
    if (!keys || !codebooks || !codes)
        return fail(LOOKAT_ERR_NULL, "keys, codebooks and codes must be non-NULL");
    if (code_stride_bh < N * shape->m)
        return fail(LOOKAT_ERR_SHAPE, "code_stride_bh=%lld is smaller than N*m=%lld", (long long)code_stride_bh,
                    (long long)(N * shape->m));
    if (!aligned16(keys) || !aligned16(codebooks))
        return fail(LOOKAT_ERR_ALIGN, "keys and codebooks must be 16-byte aligned");
    const int64_t rows = (int64_t)shape->B * N;
    if ((rows + kEncThreads - 1) / kEncThreads > 0x7fffffffLL || shape->H > 65535 || shape->m > 65535)
        return fail(LOOKAT_ERR_UNSUPPORTED, "B*N=%lld keys per head exceed one launch", (long long)rows);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Few keys per head (a decode step appends one per sequence): spread the centroids over
    // the threads.  Many keys (prefill): one thread per key.  The crossover is where the
    // thread-per-key grid reaches a few workgroups per compute unit.
    const int64_t per_key_blocks = (rows + kEncThreads - 1) / kEncThreads * shape->m * shape->H;
    bool done = false;
    // From a few 32-key blocks per head upwards the filter kernel is the fast path; the environment
    // variable LOOKAT_ENCODE_EXACT=1 forces the plain exact kernels (same codes, for comparison runs).
    const char *exact_env = getenv("LOOKAT_ENCODE_EXACT");
    const bool exact_only = exact_env && exact_env[0] == '1';
    if (!exact_only && rows >= 64)
        done = launch_encode_filter(shape, N, keys, key_dtype, codebooks, codes, code_stride_bh, st);
    if (!done && per_key_blocks < 1024 && (rows + kEncFewKeys - 1) / kEncFewKeys <= 0x7fffffffLL) {
        done = (key_dtype == LOOKAT_F16)
                   ? launch_encode_few<__half>(shape, N, keys, codebooks, codes, code_stride_bh, st)
                   : launch_encode_few<float>(shape, N, keys, codebooks, codes, code_stride_bh, st);
    }
    if (!done) {
        if (key_dtype == LOOKAT_F16)
            launch_encode<__half>(shape, N, keys, codebooks, codes, code_stride_bh, st);
        else
            launch_encode<float>(shape, N, keys, codebooks, codes, code_stride_bh, st);
    }
    return check_launch("lookat_encode_keys");
}
