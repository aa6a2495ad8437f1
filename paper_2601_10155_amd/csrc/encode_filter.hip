// Key encoding (paper Sec. 3.4, "Encoding") for many keys per head: an fp32 matrix-core filter
// in front of the exact fp64 rule.
//
// The code of a key sub-vector k is argmin_c d(k, C[c]) with d evaluated in fp64, one rounding per
// subtract / multiply / add, coordinates ascending, lowest index on ties.  Evaluating d for all 256
// centroids costs 3 fp64 operations per coordinate and centroid.  Here the 256 candidates are
// first ranked with
//     a_c = |C[c]|^2 - 2 k.C[c]        ( = d_c - |k|^2 up to rounding )
// computed by v_mfma_f32_32x32x2_f32 (rows = 32 centroids, columns = 32 keys, the norm as the
// accumulator's initial value).  Each lane keeps the smallest and second smallest a_c of its key.
// If they are further apart than twice a bound on |a_c - (exact d_c - |k|^2)|, the smallest one
// is the unique exact argmin and nothing else is evaluated.  Otherwise (near ties, exact ties,
// NaN or infinite inputs: about one sub-vector in a thousand on the workloads here) the wavefront
// evaluates the exact rule for that key over all 256 centroids.  Either way the code is the one
// the exact scan produces, bit for bit.
//
// Error bound.  a_c is an fp32 sum of d_sub + 1 terms whose magnitudes add up to at most
// S = |k|^2 + 2 max_c |C[c]|^2 (since 2|k.C| <= |k|^2 + |C|^2).  With at most 2^-23 relative
// error per accumulation step (round-to-nearest would give 2^-24) and the fp32 rounding of the
// norms, |a_c - exact| <= (d_sub + 2) 2^-22 S.  The threshold used is twice that again, plus
// 1e-30 for flushed denormals; infinite or NaN S sends the key to the exact rule.
//
// This translation unit must be compiled with -ffp-contract=off (the exact rule).
#include "common.h"

#pragma clang fp contract(off)

namespace lookat {

typedef float ef_v16f __attribute__((ext_vector_type(16)));
typedef float ef_v4f __attribute__((ext_vector_type(4)));

constexpr int kEfThreads = 256;
constexpr int kEfWaves = kEfThreads / kWave;

template <typename T>
__device__ __forceinline__ float ef_to_f32(T v);
template <>
__device__ __forceinline__ float ef_to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float ef_to_f32<__half>(__half v) { return __half2float(v); }

// N consecutive elements, fetched in the widest pieces their alignment allows (the start is a
// multiple of N elements from a 16-byte aligned row).
template <typename T, int N>
__device__ __forceinline__ void ef_load(const T *src, T (&out)[N])
{
    constexpr int BYTES = N * (int)sizeof(T);
    constexpr int CH = BYTES >= 16 ? 16 : BYTES;   // 4, 8 or 16
    typedef unsigned int chunk_t __attribute__((ext_vector_type(CH / 4)));
    chunk_t tmp[BYTES / CH];
#pragma unroll
    for (int k = 0; k < BYTES / CH; ++k)
        tmp[k] = reinterpret_cast<const chunk_t *>(src)[k];
    __builtin_memcpy(out, tmp, BYTES);
}

// Total order that reproduces the serial scan of the exact rule: smaller distance first, then
// smaller index; a NaN distance orders above everything except at centroid 0, where it orders
// below everything (the scan starts from centroid 0 and nothing compares below a NaN).
__device__ __forceinline__ uint64_t ef_order_key(double d, int c)
{
    if (d != d)
        return c == 0 ? 0ull : ~0ull;
    return (uint64_t)__double_as_longlong(d);
}

// grid = (splits, m, H); one wavefront = one (head, subspace) codebook held in registers and a
// strided share of the head's 32-key blocks.
template <typename KT, int DSUB>
__global__ __launch_bounds__(kEfThreads, 2) void encode_filter_kernel(const KT *__restrict__ keys,
                                                                   const float *__restrict__ codebooks,
                                                                   uint8_t *__restrict__ codes,
                                                                   int64_t code_stride_bh, int B, int H, int64_t N,
                                                                   int d_k, int m, int64_t blocks_per_bh)
{
    constexpr int DH = DSUB / 2;   // coordinates per lane half: lanes 0..31 take 0..DH-1, lanes 32..63 the rest
    static_assert(DSUB >= 4 && DSUB % 4 == 0, "two coordinates per lane half and matrix instruction");
    __shared__ __align__(16) float cn_s[kEfWaves][kCentroids];

    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int col = lane & 31;   // centroid within a 32-row tile (operand A), key within a block (operand B)
    const int h2 = lane >> 5;

    // ---- operand A for the 8 row tiles: -2 C[32t + col][h2*DH + mm]; squared norms to LDS ----
    const float *cb = codebooks + ((int64_t)h * m + i) * kCentroids * DSUB;
    float A[8][DH];
    float cnmax = 0.f;
    bool bad_norm = false;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const float *src = cb + (int64_t)(32 * t + col) * DSUB + h2 * DH;
        float part = 0.f;
#pragma unroll
        for (int mm = 0; mm < DH; mm += 2) {
            const float2 v = *reinterpret_cast<const float2 *>(src + mm);
            A[t][mm] = -2.f * v.x;
            A[t][mm + 1] = -2.f * v.y;
            part = part + v.x * v.x;
            part = part + v.y * v.y;
        }
        float mine, other;
        lanes_xor32(part, mine, other);
        const float cn = mine + other;
        if (h2 == 0)
            cn_s[wave][32 * t + col] = cn;
        cnmax = fmaxf(cnmax, cn);
        bad_norm |= !(cn < INFINITY);   // NaN or infinite centroid: min/median below would skip its score
    }
    cnmax = wave_max(cnmax);
    if (__ballot(bad_norm))
        cnmax = NAN;   // no key is ever "decided" by the filter: every one takes the exact rule
    __syncthreads();   // the norms are in LDS

    const float bound_factor = (float)(DSUB + 2) * 0x1p-21f;   // twice (d_sub + 2) 2^-22
    const int64_t total_blocks = (int64_t)B * blocks_per_bh;
    const ef_v4f *cn4 = reinterpret_cast<const ef_v4f *>(cn_s[wave]);

    for (int64_t kb = (int64_t)blockIdx.x * kEfWaves + wave; kb < total_blocks; kb += (int64_t)gridDim.x * kEfWaves) {
        const int64_t b = kb / blocks_per_bh;
        const int64_t n = (kb % blocks_per_bh) * 32 + col;
        const bool valid = n < N;
        const int64_t bh = b * H + h;
        // ---- operand B: this lane's half of key n's sub-vector ----
        float kv[DH];
        float kpart = 0.f;
        {
            const KT *src = keys + (bh * N + (valid ? n : 0)) * d_k + (int64_t)i * DSUB + h2 * DH;
            KT raw[DH];
            ef_load<KT, DH>(src, raw);
#pragma unroll
            for (int mm = 0; mm < DH; ++mm) {
                kv[mm] = valid ? ef_to_f32<KT>(raw[mm]) : 0.f;
                kpart = kpart + kv[mm] * kv[mm];
            }
        }
        float best = INFINITY, second = INFINITY;
        int idx = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            ef_v16f acc;
#pragma unroll
            for (int q = 0; q < 4; ++q) {   // rows 8q + 4*h2 + (0..3) of the tile start at their norms
                const ef_v4f c4 = cn4[(32 * t + 8 * q + 4 * h2) / 4];
                acc[4 * q] = c4[0];
                acc[4 * q + 1] = c4[1];
                acc[4 * q + 2] = c4[2];
                acc[4 * q + 3] = c4[3];
            }
#pragma unroll
            for (int mm = 0; mm < DH; ++mm)   // instruction mm contracts coordinates (mm, DH + mm)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(A[t][mm], kv[mm], acc, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float x = acc[r];
                idx = (x < best) ? (32 * t + 8 * (r / 4) + (r % 4)) : idx;   // + 4*h2, added below
                second = __builtin_amdgcn_fmed3f(best, x, second);          // best <= second: the middle one
                best = fminf(best, x);
            }
            __builtin_amdgcn_sched_barrier(0);   // one tile's accumulators at a time
        }
        idx += 4 * h2;
        // ---- merge the two lane halves (they hold disjoint centroids of the same key) ----
        float kmine, kother, bmine, bother, smine, sother;
        lanes_xor32(kpart, kmine, kother);
        lanes_xor32(best, bmine, bother);
        lanes_xor32(second, smine, sother);
        const int oidx = __shfl_xor(idx, 32);
        const float kn = kmine + kother;
        const float nbest = fminf(bmine, bother);
        const float nsecond = fminf(fmaxf(bmine, bother), fminf(smine, sother));
        int code = (bother < bmine) ? oidx : idx;
        const float tau = bound_factor * (kn + 2.f * cnmax) * 1.001f + 1e-30f;
        const bool unique = (nsecond - nbest) > tau;   // false for NaN / inf on either side

        // ---- exact rule for the keys the filter could not decide ----
        uint64_t todo = __ballot(valid && !unique && h2 == 0);
        while (todo) {
            const int l = __builtin_amdgcn_readfirstlane((int)__builtin_ctzll(todo));
            todo &= todo - 1;
            // lanes 0..31 accumulate coordinates 0..DH-1 of their 8 centroids, hand the partial sums
            // to lanes 32..63, which add coordinates DH..DSUB-1: one chain, coordinates ascending.
            // Rare path: operands are re-read from memory in rolled loops, so it costs no registers.
            const KT *xsrc = keys + (bh * N + ((kb % blocks_per_bh) * 32 + l)) * d_k + (int64_t)i * DSUB + h2 * DH;
            uint64_t okey = ~0ull;
            int oc = kCentroids;
#pragma unroll 1
            for (int t = 0; t < 8; ++t) {
                const float *csrc = cb + (int64_t)(32 * t + col) * DSUB + h2 * DH;
                double part = 0.0;
                if (!h2) {
#pragma unroll 1
                    for (int mm = 0; mm < DH; ++mm) {
                        const double diff = (double)ef_to_f32<KT>(xsrc[mm]) - (double)csrc[mm];
                        const double sq = diff * diff;
                        part = part + sq;
                    }
                }
                const unsigned long long bits = (unsigned long long)__double_as_longlong(part);
                const unsigned long long from_lo = __shfl_xor(bits, 32);   // upper lanes receive the lower half's sum
                if (h2) {
                    double acc = __longlong_as_double((long long)from_lo);
#pragma unroll 1
                    for (int mm = 0; mm < DH; ++mm) {
                        const double diff = (double)ef_to_f32<KT>(xsrc[mm]) - (double)csrc[mm];
                        const double sq = diff * diff;
                        acc = acc + sq;
                    }
                    const int c = 32 * t + col;
                    const uint64_t k2 = ef_order_key(acc, c);
                    if (k2 < okey) {   // c ascends with t: strict '<' keeps the lowest index
                        okey = k2;
                        oc = c;
                    }
                }
            }
            // minimum over the 32 upper lanes (xor offsets below 32 stay inside the half)
#pragma unroll
            for (int o = 16; o >= 1; o >>= 1) {
                const uint64_t k2 = __shfl_xor((unsigned long long)okey, o);
                const int c2 = __shfl_xor(oc, o);
                if (k2 < okey || (k2 == okey && c2 < oc)) {
                    okey = k2;
                    oc = c2;
                }
            }
            const int exact = __shfl(oc, 32);
            if (lane == l)
                code = exact;
        }
        if (valid && h2 == 0)
            codes[bh * code_stride_bh + n * m + i] = (uint8_t)code;
    }
}

// Launches the filter encoder if the shape has an instance; returns false otherwise.
template <typename KT>
static bool launch_encode_filter_t(const lookat_shape *s, int64_t N, const void *keys, const float *codebooks,
                                   uint8_t *codes, int64_t code_stride_bh, hipStream_t st)
{
    const int d_sub = s->d_k / s->m;
    const int64_t blocks_per_bh = (N + 31) / 32;
    const int64_t total_blocks = (int64_t)s->B * blocks_per_bh;
    // enough workgroups to fill the chip several times over, and at least 8 key blocks per wavefront
    // so that loading the codebook (the price of a wavefront) is amortised
    int64_t splits = (2048 + (int64_t)s->H * s->m - 1) / ((int64_t)s->H * s->m);
    const int64_t by_work = (total_blocks + kEfWaves * 8 - 1) / (kEfWaves * 8);
    if (splits > by_work)
        splits = by_work;
    if (splits < 1)
        splits = 1;
    dim3 grid((unsigned)splits, (unsigned)s->m, (unsigned)s->H);
    dim3 block(kEfThreads);
    const KT *k = static_cast<const KT *>(keys);
#define LOOKAT_EF_CASE(D)                                                                                          \
    case D:                                                                                                        \
        hipLaunchKernelGGL((encode_filter_kernel<KT, D>), grid, block, 0, st, k, codebooks, codes, code_stride_bh, \
                           s->B, s->H, N, s->d_k, s->m, blocks_per_bh);                                            \
        return true;
    switch (d_sub) {
        LOOKAT_EF_CASE(4)
        LOOKAT_EF_CASE(8)
        LOOKAT_EF_CASE(16)
        LOOKAT_EF_CASE(32)
    default:
        return false;
    }
#undef LOOKAT_EF_CASE
}

bool launch_encode_filter(const lookat_shape *s, int64_t N, const void *keys, int key_dtype, const float *codebooks,
                          uint8_t *codes, int64_t code_stride_bh, hipStream_t st)
{
    return (key_dtype == LOOKAT_F16)
               ? launch_encode_filter_t<__half>(s, N, keys, codebooks, codes, code_stride_bh, st)
               : launch_encode_filter_t<float>(s, N, keys, codebooks, codes, code_stride_bh, st);
}

}  // namespace lookat
