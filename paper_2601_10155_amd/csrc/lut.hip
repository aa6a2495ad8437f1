// Lookup-table construction (paper Sec. 3.5, "Precomputation Lookup Tables";
// Algorithm 1, first loop): lut[b,h,t,i,c] = q[b,h,t]^(i) . C_{h,i}[c], fp32 accumulate.
#include "common.h"

namespace lookat {

constexpr int kLutThreads = kCentroids;  // one thread per centroid

template <typename QT>
__device__ __forceinline__ float to_f32(QT v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_f32<__half>(__half v) { return __half2float(v); }

// One block = one head h, one subspace i, QB consecutive queries of the flattened
// (b, t) list.  Thread c keeps centroid c of the subspace in registers and reuses it for
// every query of the block; the query sub-vectors sit in LDS and are read by all lanes
// at the same address (broadcast).  Each query's 256 table entries are written as one
// contiguous 1 KB row.
//   grid = (ceil(B*T / QB), m, H)
template <typename QT, int DSUB>
__global__ __launch_bounds__(kLutThreads) void build_lut_kernel(const QT *__restrict__ q,
                                                                const float *__restrict__ codebooks,
                                                                float *__restrict__ lut, int B, int H, int T, int d_k,
                                                                int m, int QB)
{
    extern __shared__ float q_s[];  // [QB][DSUB]
    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int c = threadIdx.x;
    const int64_t nq = (int64_t)B * T;
    const int64_t q0 = (int64_t)blockIdx.x * QB;

    for (int e = threadIdx.x; e < QB * DSUB; e += kLutThreads) {
        const int64_t qi = q0 + e / DSUB;
        float v = 0.f;
        if (qi < nq) {
            const int64_t b = qi / T, t = qi % T;
            v = to_f32<QT>(q[((b * H + h) * T + t) * d_k + (int64_t)i * DSUB + e % DSUB]);
        }
        q_s[e] = v;
    }

    float row[DSUB];
    const float *src = codebooks + (((int64_t)h * m + i) * kCentroids + c) * DSUB;
#pragma unroll
    for (int j = 0; j < DSUB; ++j)
        row[j] = src[j];
    __syncthreads();

    for (int k = 0; k < QB; ++k) {
        const int64_t qi = q0 + k;
        if (qi >= nq)
            break;
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < DSUB; ++j)
            acc = fmaf(q_s[k * DSUB + j], row[j], acc);
        const int64_t b = qi / T, t = qi % T;
        lut[((((b * H + h) * T + t) * m) + i) * kCentroids + c] = acc;
    }
}

// Any d_sub: centroid row streamed from memory per query.
template <typename QT>
__global__ __launch_bounds__(kLutThreads) void build_lut_generic_kernel(const QT *__restrict__ q,
                                                                        const float *__restrict__ codebooks,
                                                                        float *__restrict__ lut, int B, int H, int T,
                                                                        int d_k, int m, int QB)
{
    const int d_sub = d_k / m;
    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int c = threadIdx.x;
    const int64_t nq = (int64_t)B * T;
    const float *src = codebooks + (((int64_t)h * m + i) * kCentroids + c) * d_sub;
    for (int k = 0; k < QB; ++k) {
        const int64_t qi = (int64_t)blockIdx.x * QB + k;
        if (qi >= nq)
            break;
        const int64_t b = qi / T, t = qi % T;
        const QT *qv = q + ((b * H + h) * T + t) * d_k + (int64_t)i * d_sub;
        float acc = 0.f;
        for (int j = 0; j < d_sub; ++j)
            acc = fmaf(to_f32<QT>(qv[j]), src[j], acc);
        lut[((((b * H + h) * T + t) * m) + i) * kCentroids + c] = acc;
    }
}

// ---- many queries per head: the table build is a dense contraction -> matrix cores ------
// Per (head h, subspace i):  LUT[r][c] = sum_j Q[r][j] * C[c][j]  with r over the B*T queries
// of the head, c over the 256 centroids, j over d_sub: an [R x d_sub] . [d_sub x 256] product.
// One wavefront owns 32-query tiles and keeps the whole [d_sub x 256] codebook slice in
// registers as MFMA B-fragments; per tile it issues 8 column blocks x d_sub/2 steps of
// v_mfma_f32_32x32x2_f32 (fp32 in, fp32 accumulate: same accuracy class as the vector kernel)
// and streams the 32 x 256 fp32 results out through an LDS transpose, 16 bytes per lane and 512
// contiguous bytes per half-wavefront.  The kernel is bound by that output stream (d_sub*2 flops per 4 bytes
// written), not by the matrix cores.  NTS = 1 writes the tables with non-temporal stores: a table set far
// larger than the last-level cache is read back from HBM by its consumer whatever the stores do, and
// stores that do not allocate cache lines reach 5.7-5.8 TB/s where plain ones reach 5.0-5.1 (workload
// of 4.3 GB of tables); small table sets keep plain stores so that the consumer finds them in cache.
//   fragment layout of the 32x32x2 MFMA: A[row = lane%32][k = lane/32], B[k = lane/32][col = lane%32],
//   D[row = 8*(r/4) + 4*(lane/32) + r%4][col = lane%32] for accumulator register r = 0..15.
typedef float v16f __attribute__((ext_vector_type(16)));
constexpr int kMfmaWaves = 4;

typedef float lut_v4f __attribute__((ext_vector_type(4)));

template <typename QT, int DSUB, int NTS>
__global__ __launch_bounds__(kMfmaWaves *kWave) void build_lut_mfma_kernel(const QT *__restrict__ q,
                                                                           const float *__restrict__ codebooks,
                                                                           float *__restrict__ lut, int B, int H,
                                                                           int T, int d_k, int m, int tiles_per_wave)
{
    constexpr int KS = DSUB / 2;
    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int n = lane & 31;
    const int kh = lane >> 5;
    const int64_t nq = (int64_t)B * T;
    const int64_t ntiles = (nq + 31) / 32;
    constexpr int kStageStride = 128;       // floats per staged query row: 4 wavefronts x 16 KB = the 64 KB of static LDS
    __shared__ __align__(16) float stage_s[kMfmaWaves][32 * kStageStride];
    float *stage = stage_s[wave];

    float bfrag[8][KS];
    {
        const float *cb = codebooks + ((int64_t)h * m + i) * kCentroids * DSUB;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
#pragma unroll
            for (int s = 0; s < KS; ++s)
                bfrag[nt][s] = cb[(nt * 32 + n) * DSUB + 2 * s + kh];
    }

    // Tiles are taken four at a time: the query fragments of the four are loaded together, then the
    // four are computed and stored.  Loads and stores share one in-order counter on this chip, so
    // every wait for a load also waits for all stores issued before it (32 KB of table rows per tile
    // and wavefront): with one load phase per four tiles that drain is paid a quarter as often.
    constexpr int kChunk = 4;
    const int64_t tile0 = ((int64_t)blockIdx.x * kMfmaWaves + wave) * tiles_per_wave;
    for (int it0 = 0; it0 < tiles_per_wave && tile0 + it0 < ntiles; it0 += kChunk) {
      float afr[kChunk][KS];
#pragma unroll
      for (int c = 0; c < kChunk; ++c) {
          const int64_t r = (tile0 + it0 + c) * 32 + n;
          const bool live = (it0 + c < tiles_per_wave) && (r < nq);
          const int64_t b = live ? r / T : 0, t = live ? r % T : 0;
          const QT *src = q + ((b * H + h) * T + t) * d_k + (int64_t)i * DSUB + kh;
#pragma unroll
          for (int s = 0; s < KS; ++s)
              afr[c][s] = live ? to_f32<QT>(src[2 * s]) : 0.f;
      }
#pragma unroll
      for (int c = 0; c < kChunk; ++c) {
        const int64_t tile = tile0 + it0 + c;
        if (it0 + c >= tiles_per_wave || tile >= ntiles)
            break;
        const float(&afrag)[KS] = afr[c];
        // The accumulator layout gives a lane one column (centroid) and 16 rows (queries): stored
        // directly, every store instruction would write 4 bytes per lane (two 128-byte pieces per
        // wavefront), and the kernel is then limited by store-instruction issue, not by HBM.  So the
        // results cross LDS: four column blocks (128 centroids) of the 32 queries are written as
        // [query][128] and read back 16 bytes per lane, 512 contiguous bytes of a table row per
        // half-wavefront, and stored with 16-byte stores.
        const int64_t r0 = tile * 32;
        const int64_t b0 = r0 / T;
        const int t0 = (int)(r0 % T);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const int nt = 4 * half + nb;
                v16f acc;
#pragma unroll
                for (int rr = 0; rr < 16; ++rr)
                    acc[rr] = 0.f;
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(afrag[s], bfrag[nt][s], acc, 0, 0, 0);
#pragma unroll
                for (int rr = 0; rr < 16; ++rr)
                    stage[(8 * (rr / 4) + 4 * kh + (rr % 4)) * kStageStride + nb * 32 + n] = acc[rr];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int rp = 0; rp < 16; ++rp) {
                const int row = 2 * rp + kh;                  // lanes 0..31: one query, lanes 32..63: the next
                const lut_v4f v = *reinterpret_cast<const lut_v4f *>(stage + row * kStageStride + 4 * n);
                const int rr = t0 + row;                      // position of the query within its batch entry, unwrapped
                const int64_t bq = b0 + rr / T;
                const int tq = rr % T;
                if (r0 + row < nq) {
                    float *dst = lut + ((((bq * H + h) * T + tq) * m) + i) * kCentroids + half * 128 + 4 * n;
                    if (NTS)
                        __builtin_nontemporal_store(v, reinterpret_cast<lut_v4f *>(dst));
                    else
                        *reinterpret_cast<lut_v4f *>(dst) = v;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();              // the next half overwrites the staging area
        }
      }
    }
}

template <typename QT>
static bool launch_build_lut_mfma(const lookat_shape *s, int T, const void *q, const float *codebooks, float *lut,
                                  hipStream_t st)
{
    const int d_sub = s->d_k / s->m;
    const int64_t nq = (int64_t)s->B * T;
    const int64_t ntiles = (nq + 31) / 32;
    // tiles per wave: reuse the codebook fragments, but keep at least four thousand workgroups
    int tpw = 1;
    while (tpw < 16 && (ntiles / (kMfmaWaves * tpw * 2)) * s->m * s->H >= 4096)
        tpw *= 2;
    const int64_t gx = (ntiles + (int64_t)kMfmaWaves * tpw - 1) / ((int64_t)kMfmaWaves * tpw);
    if (gx > 0x7fffffffLL)
        return false;
    dim3 grid((unsigned)gx, (unsigned)s->m, (unsigned)s->H);
    dim3 block(kMfmaWaves * kWave);
    const QT *qp = static_cast<const QT *>(q);
    // tables beyond the last-level cache (256 MB) bypass it on the way out
    const bool nts = (int64_t)nq * s->H * s->m * kCentroids * (int64_t)sizeof(float) > (int64_t)256 << 20;
#define LOOKAT_LUTM_CASE(D)                                                                                       \
    case D:                                                                                                       \
        if (nts)                                                                                                  \
            hipLaunchKernelGGL((build_lut_mfma_kernel<QT, D, 1>), grid, block, 0, st, qp, codebooks, lut, s->B,   \
                               s->H, T, s->d_k, s->m, tpw);                                                       \
        else                                                                                                      \
            hipLaunchKernelGGL((build_lut_mfma_kernel<QT, D, 0>), grid, block, 0, st, qp, codebooks, lut, s->B,   \
                               s->H, T, s->d_k, s->m, tpw);                                                       \
        return true;
    switch (d_sub) {
        LOOKAT_LUTM_CASE(2)
        LOOKAT_LUTM_CASE(4)
        LOOKAT_LUTM_CASE(8)
        LOOKAT_LUTM_CASE(16)
    default:
        return false;   // fragments would not fit the register file: vector kernel
    }
#undef LOOKAT_LUTM_CASE
}

template <typename QT>
static void launch_build_lut(const lookat_shape *s, int T, const void *q, const float *codebooks, float *lut,
                             hipStream_t st)
{
    const int d_sub = s->d_k / s->m;
    const int64_t nq = (int64_t)s->B * T;
    // queries per block: reuse the centroid registers, but keep >= ~1024 blocks in flight
    int QB = 1;
    while (QB < 16 && (nq / (QB * 2)) * s->m * s->H >= 1024)
        QB *= 2;
    dim3 grid((unsigned)((nq + QB - 1) / QB), (unsigned)s->m, (unsigned)s->H);
    dim3 block(kLutThreads);
    const QT *qp = static_cast<const QT *>(q);
#define LOOKAT_LUT_CASE(D)                                                                                         \
    case D:                                                                                                        \
        hipLaunchKernelGGL((build_lut_kernel<QT, D>), grid, block, (size_t)QB * D * sizeof(float), st, qp,         \
                           codebooks, lut, s->B, s->H, T, s->d_k, s->m, QB);                                       \
        break;
    switch (d_sub) {
        LOOKAT_LUT_CASE(1)
        LOOKAT_LUT_CASE(2)
        LOOKAT_LUT_CASE(4)
        LOOKAT_LUT_CASE(8)
        LOOKAT_LUT_CASE(16)
        LOOKAT_LUT_CASE(32)
        LOOKAT_LUT_CASE(64)
    default:
        hipLaunchKernelGGL((build_lut_generic_kernel<QT>), grid, block, 0, st, qp, codebooks, lut, s->B, s->H, T,
                           s->d_k, s->m, QB);
        break;
    }
#undef LOOKAT_LUT_CASE
}

}  // namespace lookat

extern "C" int lookat_build_lut(const lookat_shape *shape, int32_t T, const void *q, lookat_dtype q_dtype,
                                const float *codebooks, float *lut, void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (T <= 0)
        return fail(LOOKAT_ERR_SHAPE, "T=%d must be positive", T);
    if (q_dtype != LOOKAT_F16 && q_dtype != LOOKAT_F32)
        return fail(LOOKAT_ERR_DTYPE, "q_dtype=%d is neither LOOKAT_F16 nor LOOKAT_F32", q_dtype);
    if (!q || !codebooks || !lut)
        return fail(LOOKAT_ERR_NULL, "q, codebooks and lut must be non-NULL");
    if (!aligned16(q) || !aligned16(codebooks) || !aligned16(lut))
        return fail(LOOKAT_ERR_ALIGN, "q, codebooks and lut must be 16-byte aligned");
    if ((int64_t)shape->B * T > 0x7fffffffLL || shape->H > 65535)
        return fail(LOOKAT_ERR_UNSUPPORTED, "B*T or H too large for one launch");
    hipStream_t st = static_cast<hipStream_t>(stream);
    // From 256 queries per head on, the build is a dense [B*T x d_sub].[d_sub x 256] contraction
    // per (head, subspace) and runs on the matrix cores; below that the 32-row MFMA tiles would be
    // mostly padding and the vector kernel is used.
    bool done = false;
    if ((int64_t)shape->B * T >= 256)
        done = (q_dtype == LOOKAT_F16) ? launch_build_lut_mfma<__half>(shape, T, q, codebooks, lut, st)
                                       : launch_build_lut_mfma<float>(shape, T, q, codebooks, lut, st);
    if (!done) {
        if (q_dtype == LOOKAT_F16)
            launch_build_lut<__half>(shape, T, q, codebooks, lut, st);
        else
            launch_build_lut<float>(shape, T, q, codebooks, lut, st);
    }
    return check_launch("lookat_build_lut");
}
