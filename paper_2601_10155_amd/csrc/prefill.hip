// Causal lookup-and-sum scoring for a block of T queries (prefill): every query builds its
// lookup tables (paper Sec. 3.5, "Precomputation Lookup Tables") and scores the coded keys
// it may see (Sec. 3.5, "Lookup and Sum"; Algorithm 1, second loop), without the tables ever
// leaving the chip:
//     scores[b,h,t,l] = sum_i LUT_{b,h,t,i}[codes[b,h,l,i]]   for l <= t + (L - T),  else -inf.
//
// Shape of the computation on gfx950
//   * one workgroup (512 threads) = one (b,h) and kPfGroup consecutive tiles of TQ = 4 queries;
//     two workgroups fit a compute unit (64 KB of tables each), so one builds tables on the
//     vector ALU while the other gathers from LDS;
//   * the tables of a tile live in LDS as lut_s[i][c][4] (fp32): the four queries' entries of one
//     (subspace, centroid) are adjacent, so ONE 16-byte LDS read per (key, subspace) serves four
//     queries.  Against a [query][i][c] layout with 4-byte gathers this is a quarter of the LDS
//     instructions, and the 16-byte stride spreads a pass of 8 lanes over all banks;
//   * the head's codebook is held in registers across the workgroup's tiles (thread p owns the
//     (subspace, centroid) pairs p, p+512, ...), so a tile's tables cost d_sub FMAs per entry and
//     no codebook traffic.  With 4 queries per tile the contraction is 4 wide: a 32x32 or 16x16
//     MFMA tile would be 75-87% padding and fp32 MFMA has no rate advantage over the vector
//     ALU, so this step stays on the vector ALU;
//   * the scoring loop is bound by LDS read bandwidth (4 bytes per (query, key, subspace)) and by
//     the scores written (4 bytes per (query, key)).
#include "common.h"

namespace lookat {

constexpr int kPfThreads = 512;
constexpr int kPfTQ = 4;      // queries per tile
constexpr int kPfGroup = 8;   // query tiles per workgroup (codebook registers reused)

typedef unsigned int pf_v4u __attribute__((ext_vector_type(4)));
typedef unsigned int pf_v2u __attribute__((ext_vector_type(2)));

template <typename QT>
__device__ __forceinline__ float pf_to_f32(QT v);
template <>
__device__ __forceinline__ float pf_to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float pf_to_f32<__half>(__half v) { return __half2float(v); }

struct PrefillArgs {
    const void *q;            // [BH, T, d_k]
    const float *codebooks;   // [H, m, 256, d_sub]
    const uint8_t *codes;     // (bh, l, i) at bh*code_stride + l*m + i
    float *scores;            // [BH, T, L]
    int64_t code_stride;
    int64_t L;
    int T;
    int H;
    int tiles;                // ceil(T / 4)
    int BH;
    int groups;               // ceil(tiles / kPfGroup)
};

template <int M>
struct PfCodes {
    uint32_t w[(M + 3) / 4];
    __device__ __forceinline__ void load(const uint8_t *cp)
    {
        if constexpr (M == 2) {
            w[0] = *reinterpret_cast<const uint16_t *>(cp);
        } else if constexpr (M == 4) {
            w[0] = *reinterpret_cast<const uint32_t *>(cp);
        } else if constexpr (M == 8) {
            const pf_v2u t = *reinterpret_cast<const pf_v2u *>(cp);
            w[0] = t.x;
            w[1] = t.y;
        } else {
            const pf_v4u t = *reinterpret_cast<const pf_v4u *>(cp);
            w[0] = t.x;
            w[1] = t.y;
            w[2] = t.z;
            w[3] = t.w;
        }
    }
    __device__ __forceinline__ uint32_t byte(int i) const { return (w[i / 4] >> (8 * (i % 4))) & 0xffu; }
};

// grid = 8 * ceil(BH / 8) * ceil(tiles / kPfGroup) workgroups, mapped to ((b,h), tile group) below.
template <typename QT, int DK, int M>
__global__ __launch_bounds__(kPfThreads, 4) void score_prefill_kernel(const PrefillArgs a)
{
    constexpr int TQ = kPfTQ;
    constexpr int DSUB = DK / M;
    constexpr int PAIRS = M * kCentroids;                          // (subspace, centroid) pairs
    constexpr int PP = (PAIRS + kPfThreads - 1) / kPfThreads;      // pairs per thread
    constexpr int GB = M < 4 ? M : 4;                              // gathers in flight per key
    extern __shared__ __align__(16) float smem[];
    float *lut_s = smem;                      // [M][256][TQ]
    float *q_s = smem + PAIRS * TQ;           // [TQ][DK]

    // Workgroup ids are dealt round-robin to the 8 dies, each with its own 4 MB L2.  (b,h) pairs
    // are assigned so that a die only ever sees the heads congruent to its index mod 8: its L2
    // then holds a few heads' codebooks (128 KB each at d_k = 128) instead of cycling through all
    // of them.  Within a die, late (long) tile groups come first.
    const int xcd = blockIdx.x % 8;
    const int slot = blockIdx.x / 8;
    const int bh_per_xcd = (a.BH + 7) / 8;
    const int bh = (slot % bh_per_xcd) * 8 + xcd;
    const int group = a.groups - 1 - slot / bh_per_xcd;
    if (bh >= a.BH)
        return;
    const int h = bh % a.H;
    const int tid = threadIdx.x;
    const int64_t off = a.L - a.T;            // query t sits at position t + off
    const QT *qg = static_cast<const QT *>(a.q) + (int64_t)bh * a.T * DK;
    const uint8_t *codes_bh = a.codes + (int64_t)bh * a.code_stride;
    float *scores_bh = a.scores + (int64_t)bh * a.T * a.L;

    // codebook rows of this thread's (subspace, centroid) pairs, kept for all tiles
    float row[PP][DSUB];
#pragma unroll
    for (int k = 0; k < PP; ++k) {
        const int p = tid + k * kPfThreads;
        if (p < PAIRS) {
            const float4 *src = reinterpret_cast<const float4 *>(a.codebooks + ((int64_t)h * PAIRS + p) * DSUB);
#pragma unroll
            for (int j4 = 0; j4 < DSUB / 4; ++j4) {
                const float4 v = src[j4];
                row[k][4 * j4] = v.x;
                row[k][4 * j4 + 1] = v.y;
                row[k][4 * j4 + 2] = v.z;
                row[k][4 * j4 + 3] = v.w;
            }
        }
    }

    for (int g = 0; g < kPfGroup; ++g) {
        const int tile = group * kPfGroup + (kPfGroup - 1 - g);
        if (tile >= a.tiles)
            continue;
        const int t0 = tile * TQ;
        const int64_t vis_last = t0 + TQ - 1 + off;                     // last key any query of the tile sees
        const int64_t kmax = (vis_last + 1 < a.L) ? vis_last + 1 : a.L;

        __syncthreads();   // the previous tile's readers are done with lut_s / q_s
        for (int e = tid; e < TQ * DK; e += kPfThreads) {
            const int t = t0 + e / DK;
            q_s[e] = (t < a.T) ? pf_to_f32<QT>(qg[(int64_t)t * DK + e % DK]) : 0.f;
        }
        // codes of this thread's first key: requested now, needed after the table build
        PfCodes<M> kc;
        if (tid < kmax)
            kc.load(codes_bh + (int64_t)tid * M);
        __syncthreads();

        // ---- tables of the tile: lut_s[(i*256 + c)*4 + t] = q[t]^(i) . C_i[c], j ascending ----
#pragma unroll
        for (int k = 0; k < PP; ++k) {
            const int p = tid + k * kPfThreads;
            if (p < PAIRS) {
                const int i = p / kCentroids;   // uniform over the wavefront: q_s reads are broadcasts
                float acc[TQ];
#pragma unroll
                for (int t = 0; t < TQ; ++t) {
                    const float4 *qv = reinterpret_cast<const float4 *>(q_s + t * DK + i * DSUB);
                    acc[t] = 0.f;
#pragma unroll
                    for (int j4 = 0; j4 < DSUB / 4; ++j4) {
                        const float4 x = qv[j4];
                        acc[t] = fmaf(x.x, row[k][4 * j4], acc[t]);
                        acc[t] = fmaf(x.y, row[k][4 * j4 + 1], acc[t]);
                        acc[t] = fmaf(x.z, row[k][4 * j4 + 2], acc[t]);
                        acc[t] = fmaf(x.w, row[k][4 * j4 + 3], acc[t]);
                    }
                }
                *reinterpret_cast<float4 *>(lut_s + (int64_t)p * TQ) = make_float4(acc[0], acc[1], acc[2], acc[3]);
            }
        }
        __syncthreads();

        // ---- scoring: one key per thread and step, four scores per key ----
        for (int64_t l = tid; l < kmax; l += kPfThreads) {
            float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int i0 = 0; i0 < M; i0 += GB) {
                float4 v[GB];
#pragma unroll
                for (int u = 0; u < GB; ++u)
                    v[u] = *reinterpret_cast<const float4 *>(lut_s + ((i0 + u) * kCentroids + kc.byte(i0 + u)) * TQ);
#pragma unroll
                for (int u = 0; u < GB; ++u) {   // ascending subspace order, as Algorithm 1 sums
                    s.x += v[u].x;
                    s.y += v[u].y;
                    s.z += v[u].z;
                    s.w += v[u].w;
                }
            }
            const int64_t ln = l + kPfThreads;
            if (ln < kmax)
                kc.load(codes_bh + ln * M);   // next key of this thread
            const float sv[TQ] = {s.x, s.y, s.z, s.w};
#pragma unroll
            for (int t = 0; t < TQ; ++t) {
                const int tq = t0 + t;
                if (tq < a.T)
                    scores_bh[(int64_t)tq * a.L + l] = (l <= tq + off) ? sv[t] : -INFINITY;
            }
        }
        // ---- keys no query of the tile may see ----
        for (int t = 0; t < TQ; ++t) {
            const int tq = t0 + t;
            if (tq >= a.T)
                break;
            for (int64_t l = kmax + tid; l < a.L; l += kPfThreads)
                scores_bh[(int64_t)tq * a.L + l] = -INFINITY;
        }
    }
}

template <typename QT, int DK, int M>
static int launch_prefill(const PrefillArgs &a0, int BH, hipStream_t st)
{
    PrefillArgs a = a0;
    a.tiles = (a.T + kPfTQ - 1) / kPfTQ;
    const size_t lds = ((size_t)M * kCentroids * kPfTQ + (size_t)kPfTQ * DK) * sizeof(float);
    auto kern = score_prefill_kernel<QT, DK, M>;
    if (lds > 64 * 1024) {
        static bool configured = false;   // per instantiation: allow more than 64 KB of dynamic LDS
        if (!configured) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess)
                return fail(LOOKAT_ERR_HIP, "lookat_score_prefill: cannot reserve %zu bytes of LDS: %s", lds,
                            hipGetErrorString(e));
            configured = true;
        }
    }
    a.BH = BH;
    a.groups = (a.tiles + kPfGroup - 1) / kPfGroup;
    dim3 grid((unsigned)((BH + 7) / 8 * 8 * a.groups));
    hipLaunchKernelGGL(kern, grid, dim3(kPfThreads), lds, st, a);
    return check_launch("lookat_score_prefill");
}

template <typename QT>
static int dispatch_prefill(const lookat_shape *s, const PrefillArgs &a, hipStream_t st)
{
    const int BH = s->B * s->H;
#define LOOKAT_PF_CASE(DK_, M_)             \
    if (s->d_k == DK_ && s->m == M_)        \
        return launch_prefill<QT, DK_, M_>(a, BH, st);
    LOOKAT_PF_CASE(64, 2)
    LOOKAT_PF_CASE(64, 4)
    LOOKAT_PF_CASE(64, 8)
    LOOKAT_PF_CASE(64, 16)
    LOOKAT_PF_CASE(128, 2)
    LOOKAT_PF_CASE(128, 4)
    LOOKAT_PF_CASE(128, 8)
    LOOKAT_PF_CASE(128, 16)
#undef LOOKAT_PF_CASE
    return fail(LOOKAT_ERR_UNSUPPORTED, "lookat_score_prefill handles d_k in {64,128} with m in {2,4,8,16}; got d_k=%d m=%d",
                s->d_k, s->m);
}

}  // namespace lookat

extern "C" int lookat_score_prefill(const lookat_shape *shape, int32_t T, int64_t L, const void *q, int q_dtype,
                                    const float *codebooks, const uint8_t *codes, int64_t code_stride_bh,
                                    float *scores, void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (T <= 0 || L < T)
        return fail(LOOKAT_ERR_SHAPE, "need 1 <= T <= L (T=%d, L=%lld)", T, (long long)L);
    if (q_dtype != LOOKAT_F16 && q_dtype != LOOKAT_F32)
        return fail(LOOKAT_ERR_DTYPE, "q_dtype=%d is neither LOOKAT_F16 nor LOOKAT_F32", q_dtype);
    if (!q || !codebooks || !codes || !scores)
        return fail(LOOKAT_ERR_NULL, "q, codebooks, codes and scores must be non-NULL");
    if (code_stride_bh < L * shape->m)
        return fail(LOOKAT_ERR_SHAPE, "code_stride_bh=%lld is smaller than L*m", (long long)code_stride_bh);
    if (!aligned16(q) || !aligned16(codebooks) || (reinterpret_cast<uintptr_t>(scores) & 3u))
        return fail(LOOKAT_ERR_ALIGN, "q and codebooks must be 16-byte aligned, scores 4-byte aligned");
    const int cvec = (shape->m == 2 || shape->m == 4 || shape->m == 8 || shape->m == 16) ? shape->m : 1;
    if ((reinterpret_cast<uintptr_t>(codes) % cvec) || (code_stride_bh % cvec))
        return fail(LOOKAT_ERR_ALIGN, "codes and code_stride_bh must be multiples of %d bytes for m=%d", cvec, shape->m);
    {
        const int64_t BHp = ((int64_t)shape->B * shape->H + 7) / 8 * 8;
        const int64_t groups = ((int64_t)(T + kPfTQ - 1) / kPfTQ + kPfGroup - 1) / kPfGroup;
        if (BHp * groups > 0x7fffffffLL)
            return fail(LOOKAT_ERR_UNSUPPORTED, "B*H*T=%lld*%d exceeds one launch", (long long)shape->B * shape->H, T);
    }
    PrefillArgs a;
    a.q = q;
    a.codebooks = codebooks;
    a.codes = codes;
    a.scores = scores;
    a.code_stride = code_stride_bh;
    a.L = L;
    a.T = T;
    a.H = shape->H;
    a.tiles = 0;
    a.BH = 0;
    a.groups = 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return (q_dtype == LOOKAT_F16) ? dispatch_prefill<__half>(shape, a, st) : dispatch_prefill<float>(shape, a, st);
}
