// Key encoding (paper Sec. 3.4, "Encoding") for many keys per head: a matrix-core filter in
// front of the exact fp64 rule.
//
// The code of a key sub-vector k is argmin_c d(k, C[c]) with d evaluated in fp64, one rounding per
// subtract / multiply / add, coordinates ascending, lowest index on ties.  Evaluating d for all 256
// centroids costs 3 fp64 operations per coordinate and centroid.  Here the 256 candidates are
// first ranked with
//     a_c = |C[c]|^2 - 2 k.C[c]        ( = d_c - |k|^2 up to rounding )
// computed on the matrix cores (rows = 32 centroids, columns = 32 keys, the norm as the
// accumulator's initial value).  Each lane keeps the smallest and second smallest a_c of its key.
// If they are further apart than twice a bound on |a_c - (exact d_c - |k|^2)|, the smallest one
// is the unique exact argmin and nothing else is evaluated.  Otherwise (near ties, exact ties,
// NaN or infinite inputs: a few sub-vectors in ten thousand on the workloads here) the wavefront
// evaluates the exact rule for that key over all 256 centroids.  Either way the code is the one
// the exact scan produces, bit for bit.
//
// Two instances of the product:
//   * fp32 keys: v_mfma_f32_32x32x2_f32 on the operands as they are.  On this chip the fp32 matrix
//     instruction shares the vector ALU's multiply-add datapath (same peak rate, and counters show
//     its busy cycles ADD to the vector instructions' instead of overlapping them);
//   * fp16 keys: v_mfma_f32_32x32x8_f16, which runs beside the vector ALU.  The keys are exact in
//     fp16; the codebook is scaled by a power of two s (largest entry near 2^13) and split into
//     two fp16 terms, -2sC = hi + lo with |(-2sC) - hi - lo| <= 2^-22 |2sC|; fp16 products are exact
//     in fp32.  The scores are then s * a_c for all centroids of the (head, subspace) alike.
//
// Error bound.  a_c is an fp32 sum of at most 2 d_sub + 1 terms whose magnitudes add up to at most
// S = |k|^2 + 2 max_c |C[c]|^2 (since 2|k.C| <= |k|^2 + |C|^2).  With at most 2^-23 relative
// error per accumulation step (round-to-nearest would give 2^-24), the fp32 rounding of the norms
// and the 2^-22 split residual, |a_c - exact| <= (2 d_sub + 4) 2^-23 S.  The threshold used is
// four times that (twice for the two candidates, twice as margin), plus 1e-30 for flushed
// denormals; an infinite or NaN S sends the key to the exact rule.
//
// This translation unit must be compiled with -ffp-contract=off (the exact rule).
#include <cstdlib>

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

// The exact rule for key `l` of the block (l uniform over the wavefront), all 64 lanes working:
// lanes 0..31 accumulate coordinates 0..DSUB/2-1 of their 8 centroids and hand the partial sums to
// lanes 32..63, which add the remaining coordinates: one chain per centroid, coordinates ascending.
// Operands are re-read from memory (the matrix fragments are scaled and split), a few centroid
// rows at a time so that the loads of a batch are in flight together.
template <typename KT, int DSUB>
__device__ __forceinline__ int ef_exact_code(const KT *key_sub, const float *cb, int col, int h2)
{
    constexpr int DH = DSUB / 2;
    constexpr int TB = (32 / DH) > 8 ? 8 : (32 / DH);   // centroid rows per batch: at most 32 registers of operands
    KT xr[DH];
    ef_load<KT, DH>(key_sub + h2 * DH, xr);
    uint64_t okey = ~0ull;
    int oc = kCentroids;
#pragma unroll 1
    for (int t0 = 0; t0 < 8; t0 += TB) {
        float cr[TB][DH];
#pragma unroll
        for (int u = 0; u < TB; ++u)
            ef_load<float, DH>(cb + (int64_t)(32 * (t0 + u) + col) * DSUB + h2 * DH, cr[u]);
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            double part = 0.0;
#pragma unroll
            for (int mm = 0; mm < DH; ++mm) {
                const double diff = (double)ef_to_f32<KT>(xr[mm]) - (double)cr[u][mm];
                const double sq = diff * diff;
                part = part + sq;
            }
            // upper lanes restart from the lower half's sum: (lower sum) + their coordinates, in order
            const unsigned long long from_lo = __shfl_xor((unsigned long long)__double_as_longlong(part), 32);
            double acc = __longlong_as_double((long long)from_lo);
#pragma unroll
            for (int mm = 0; mm < DH; ++mm) {
                const double diff = (double)ef_to_f32<KT>(xr[mm]) - (double)cr[u][mm];
                const double sq = diff * diff;
                acc = acc + sq;
            }
            if (h2) {
                const int c = 32 * (t0 + u) + col;
                const uint64_t k2 = ef_order_key(acc, c);
                if (k2 < okey) {   // c ascends with t: strict '<' keeps the lowest index
                    okey = k2;
                    oc = c;
                }
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
    return __shfl(oc, 32);
}

// Which coordinates of a sub-vector a lane feeds to the matrix instructions, and how.
//   fp32 instance: lane half h2 holds coordinates h2*DH .. h2*DH+DH-1 as floats; instruction mm
//                  contracts coordinates (mm, DH + mm).
//   fp16 instance: instruction s contracts coordinates 8s .. 8s+7; lane half h2 holds the four
//                  coordinates 8s + 4*h2 + (0..3) as packed halves (zero where >= DSUB).
template <typename KT, int DSUB>
struct EfFrag;

template <int DSUB>
struct EfFrag<float, DSUB> {
    static constexpr int DH = DSUB / 2;
    static constexpr int NI = DH;        // matrix instructions per tile
    float a[8][DH];                      // -2 C
    float k[DH];
    __device__ __forceinline__ float load_codebook(const float *cb, int col, int h2, float *cn_row, bool &bad)
    {
        float cnmax = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const float *src = cb + (int64_t)(32 * t + col) * DSUB + h2 * DH;
            float part = 0.f;
#pragma unroll
            for (int mm = 0; mm < DH; mm += 2) {
                const float2 v = *reinterpret_cast<const float2 *>(src + mm);
                a[t][mm] = -2.f * v.x;
                a[t][mm + 1] = -2.f * v.y;
                part = part + v.x * v.x;
                part = part + v.y * v.y;
            }
            float mine, other;
            lanes_xor32(part, mine, other);
            const float cn = mine + other;
            if (h2 == 0)
                cn_row[32 * t + col] = cn;
            cnmax = fmaxf(cnmax, cn);
            bad |= !(cn < INFINITY);   // NaN or infinite centroid: the min/median updates would skip its score
        }
        return wave_max(cnmax);          // scores are in units of 1: scale 1
    }
    static __device__ __forceinline__ void fetch(const float *sub, int h2, float (&raw)[DH]) { ef_load<float, DH>(sub + h2 * DH, raw); }
    __device__ __forceinline__ float score_scale() const { return 1.f; }
    typedef float raw_t[DH];
    __device__ __forceinline__ float take(const raw_t &raw, bool valid)
    {
        float kpart = 0.f;
#pragma unroll
        for (int mm = 0; mm < DH; ++mm) {
            k[mm] = valid ? raw[mm] : 0.f;
            kpart = kpart + k[mm] * k[mm];
        }
        return kpart;
    }
    __device__ __forceinline__ ef_v16f mma(int t, int s, ef_v16f acc) const
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a[t][s], k[s], acc, 0, 0, 0);
    }
};

typedef _Float16 ef_v4h __attribute__((ext_vector_type(4)));

template <int DSUB>
struct EfFrag<__half, DSUB> {
    static constexpr int NS = (DSUB + 7) / 8;   // 8-coordinate slices
    static constexpr int NI = 2 * NS;           // matrix instructions per tile: hi and lo term of each slice
    ef_v4h hi[8][NS], lo[8][NS];                // -2 s C = hi + lo
    ef_v4h k[NS];
    float scale;                                // s
    __device__ __forceinline__ float load_codebook(const float *cb, int col, int h2, float *cn_row, bool &bad)
    {
        // largest |C| of the (head, subspace) -> s = 2^(13 - exponent), so that 2sC stays below 2^15
        float cmax = 0.f;
        float v[8][NS][4];
#pragma unroll
        for (int t = 0; t < 8; ++t)
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int d0 = 8 * s + 4 * h2;
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                if (d0 < DSUB)
                    x = *reinterpret_cast<const float4 *>(cb + (int64_t)(32 * t + col) * DSUB + d0);
                v[t][s][0] = x.x;
                v[t][s][1] = x.y;
                v[t][s][2] = x.z;
                v[t][s][3] = x.w;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    cmax = fmaxf(cmax, fabsf(v[t][s][e]));
                    bad |= !(fabsf(v[t][s][e]) < INFINITY);
                }
            }
        cmax = wave_max(cmax);
        int ex = (int)((__float_as_uint(cmax) >> 23) & 0xffu) - 127;   // floor(log2(cmax)) for normal numbers
        if (cmax == 0.f)
            ex = 0;
        int se = 13 - ex;
        se = se > 100 ? 100 : (se < -100 ? -100 : se);
        scale = __uint_as_float((uint32_t)(se + 127) << 23);
        float cnmax = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float part = 0.f;
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float c = v[t][s][e];
                    part = part + c * c;
                    const float w = -2.f * scale * c;              // exact (powers of two) unless it over/underflows
                    const _Float16 wh = (_Float16)w;
                    const _Float16 wl = (_Float16)(w - (float)wh); // exact difference, then one rounding
                    hi[t][s][e] = wh;
                    lo[t][s][e] = wl;
                }
            float mine, other;
            lanes_xor32(part, mine, other);
            const float cn = mine + other;
            if (h2 == 0)
                cn_row[32 * t + col] = scale * cn;
            cnmax = fmaxf(cnmax, cn);
            bad |= !(scale * cn < INFINITY);
        }
        return wave_max(cnmax);
    }
    __device__ __forceinline__ float score_scale() const { return scale; }
    typedef uint2 raw_t[NS];
    static __device__ __forceinline__ void fetch(const __half *sub, int h2, raw_t &raw)
    {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int d0 = 8 * s + 4 * h2;
            raw[s] = (d0 < DSUB) ? *reinterpret_cast<const uint2 *>(sub + d0) : make_uint2(0u, 0u);
        }
    }
    __device__ __forceinline__ float take(const raw_t &raw, bool valid)
    {
        float kpart = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const uint2 r = valid ? raw[s] : make_uint2(0u, 0u);
            __builtin_memcpy(&k[s], &r, 8);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x = (float)k[s][e];
                kpart = kpart + x * x;
            }
        }
        return kpart;
    }
    __device__ __forceinline__ ef_v16f mma(int t, int s, ef_v16f acc) const
    {
        return (s & 1) ? __builtin_amdgcn_mfma_f32_32x32x8f16(lo[t][s >> 1], k[s >> 1], acc, 0, 0, 0)
                       : __builtin_amdgcn_mfma_f32_32x32x8f16(hi[t][s >> 1], k[s >> 1], acc, 0, 0, 0);
    }
};

// grid = (splits, m, H); one wavefront = one (head, subspace) codebook held in registers and a
// strided share of the head's 32-key blocks.
template <typename KT, int DSUB>
__global__ __launch_bounds__(kEfThreads, 2) void encode_filter_kernel(const KT *__restrict__ keys,
                                                                      const float *__restrict__ codebooks,
                                                                      uint8_t *__restrict__ codes,
                                                                      int64_t code_stride_bh, int B, int H, int64_t N,
                                                                      int d_k, int m, int64_t blocks_per_bh)
{
    static_assert(DSUB >= 4 && DSUB % 4 == 0, "fragments are four coordinates wide");
    typedef EfFrag<KT, DSUB> Frag;
    constexpr int NI = Frag::NI;
    __shared__ __align__(16) float cn_s[kEfWaves][kCentroids];

    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int col = lane & 31;   // centroid within a 32-row tile (operand A), key within a block (operand B)
    const int h2 = lane >> 5;

    // ---- operand A for the 8 row tiles; (scaled) squared norms to LDS ----
    const float *cb = codebooks + ((int64_t)h * m + i) * kCentroids * DSUB;
    Frag f;
    bool bad_norm = false;
    float cnmax = f.load_codebook(cb, col, h2, cn_s[wave], bad_norm);
    if (__ballot(bad_norm))
        cnmax = NAN;   // no key is ever "decided" by the filter: every one takes the exact rule
    __syncthreads();   // the norms are in LDS

    const float bound_factor = (float)(2 * DSUB + 4) * 0x1p-21f;   // four times (2 d_sub + 4) 2^-23
    const int64_t total_blocks = (int64_t)B * blocks_per_bh;
    const ef_v4f *cn4 = reinterpret_cast<const ef_v4f *>(cn_s[wave]);

    // The next block's key fragments are requested while the current block is scored.
    const int64_t kb_step = (int64_t)gridDim.x * kEfWaves;
    typename Frag::raw_t raw_next;
    auto fetch_keys = [&](int64_t kb) {
        const int64_t n = (kb % blocks_per_bh) * 32 + col;
        const int64_t bh = (kb / blocks_per_bh) * H + h;
        Frag::fetch(keys + (bh * N + (n < N ? n : 0)) * d_k + (int64_t)i * DSUB, h2, raw_next);
    };
    int64_t kb = (int64_t)blockIdx.x * kEfWaves + wave;
    if (kb < total_blocks)
        fetch_keys(kb);
    for (; kb < total_blocks; kb += kb_step) {
        const int64_t b = kb / blocks_per_bh;
        const int64_t n = (kb % blocks_per_bh) * 32 + col;
        const bool valid = n < N;
        const int64_t bh = b * H + h;
        // ---- operand B: this lane's part of key n's sub-vector ----
        const float kpart = f.take(raw_next, valid);
        if (kb + kb_step < total_blocks)
            fetch_keys(kb + kb_step);
        float best = INFINITY, second = INFINITY;
        int idx = 0;
        // Software pipeline over the 8 row tiles: the matrix instructions of tile t+1 are issued
        // between the min / second-min updates of tile t.  The instructions of a tile form a
        // dependent chain, and a wavefront issues in order, so without the interleave it would sit
        // idle through the chain and then do 64 vector instructions.
        auto start_tile = [&](int t, ef_v16f &acc) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {   // rows 8q + 4*h2 + (0..3) of the tile start at their norms
                const ef_v4f c4 = cn4[(32 * t + 8 * q + 4 * h2) / 4];
                acc[4 * q] = c4[0];
                acc[4 * q + 1] = c4[1];
                acc[4 * q + 2] = c4[2];
                acc[4 * q + 3] = c4[3];
            }
        };
        ef_v16f acc_cur, acc_nxt;
        start_tile(0, acc_cur);
#pragma unroll
        for (int s = 0; s < NI; ++s)
            acc_cur = f.mma(0, s, acc_cur);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (t < 7) {
                start_tile(t + 1, acc_nxt);
#pragma unroll
                for (int s = 0; s < NI; ++s)
                    acc_nxt = f.mma(t + 1, s, acc_nxt);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float x = acc_cur[r];
                const bool lt = x < best;
                idx = lt ? (32 * t + 8 * (r / 4) + (r % 4)) : idx;   // + 4*h2, added below
                second = __builtin_amdgcn_fmed3f(best, x, second);  // best <= second: the middle one
                best = lt ? x : best;   // a select on the same compare: fminf would add a NaN-quieting instruction
            }
            if (t < 7) {
                // NI groups of (1 matrix instruction, 64/NI vector instructions)
#pragma unroll
                for (int g = 0; g < NI; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, (64 + NI - 1) / NI, 0);
                }
            }
            acc_cur = acc_nxt;
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
        const float tau = f.score_scale() * (bound_factor * (kn + 2.f * cnmax) * 1.001f) + 1e-30f;
        const bool unique = (nsecond - nbest) > tau;   // false for NaN / inf on either side

        // ---- exact rule for the keys the filter could not decide ----
        uint64_t todo = __ballot(valid && !unique && h2 == 0);
        while (todo) {
            const int l = __builtin_amdgcn_readfirstlane((int)__builtin_ctzll(todo));
            todo &= todo - 1;
            const KT *key_sub = keys + (bh * N + ((kb % blocks_per_bh) * 32 + l)) * d_k + (int64_t)i * DSUB;
            const int exact = ef_exact_code<KT, DSUB>(key_sub, cb, col, h2);
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
