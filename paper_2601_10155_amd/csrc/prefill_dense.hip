// Causal scoring of a block of T queries against coded keys (paper Sec. 3.5, "Lookup and Sum", applied to
// every query position) when T is large: the same scores as prefill.hip's lookup-and-sum kernel,
//     scores[b,h,t,l] = sum_i LUT_{b,h,t,i}[codes[b,h,l,i]] = sum_i q_t^(i) . C_i[codes_l[i]],
// evaluated in the second form.  With many queries per key the sum over subspaces of table look-ups IS a
// dense contraction  [T queries x d_k] . [d_k x keys]  against the keys' centroids, and on this chip it
// belongs on the matrix cores: a look-up costs an LDS gather and four vector adds per (4 queries, key,
// subspace), the matrix cores do the same 4 x d_sub multiply-adds in a fraction of an instruction, and the
// kernel becomes bound by the one thing that cannot be avoided, the T x L scores it writes.  Nothing leaves
// the compressed domain in memory: keys are read as codes, their centroids are fetched by code from the
// codebook (L2-resident, 128 KB per head at d_k = 128) once per key and kept in registers as the
// stationary matrix operand; no table and no decoded key is written anywhere.
//
// Shape of the computation
//   * one workgroup (4 wavefronts) owns a panel of 128 keys of one (b,h) and writes that panel's column
//     strip of all T score rows: -inf for the queries that cannot see the panel, scores for the others.
//     Every workgroup of a launch writes the same number of bytes; the matrix work differs (early panels
//     are seen by more queries) and is a small part of the time.
//   * wavefront w holds keys 32w .. 32w+31 of the panel as the B operand of v_mfma_f32_32x32x16_f16: per
//     16-coordinate step, lane (key n, half g) fetches coordinates 16s+8g .. +7 of the centroids its key's codes
//     select (two 16-byte pieces of fp32 codebook rows), scales by a power of two chosen per wavefront so that the
//     largest fetched entry sits near 2^13, and splits the result into two fp16 terms, hi = fp16(w) and
//     lo = fp16((w - hi) * 2^11): hi + lo * 2^-11 carries 22 bits of w, and fp16 x fp16 products are exact in
//     the fp32 accumulators.  Two accumulator sets (hi and lo terms) are combined when a tile is finished.
//   * queries are taken in tiles of 32 (the A operand): a tile (8 KB of fp16, contiguous in memory) is
//     staged in LDS by the whole workgroup, rows padded by 16 bytes so that the 16-byte operand reads of
//     sixteen lanes fall on distinct banks; the tile after the next is requested while the current one is
//     multiplied and written to the other buffer a step later.
//   * a tile's 32 x 128 results cross LDS once more so that they leave as 16-byte non-temporal stores, 512
//     contiguous bytes of a score row per half-wavefront (stored straight from the accumulators a store
//     instruction would write 4 bytes per lane).  The causal mask is applied on the way into LDS.
//   * loads a wavefront waits for are issued before the stores of the same step: loads and stores share one
//     in-order counter, and a wait for a load issued behind stores would wait for the stores as well.  One
//     workgroup barrier per tile: the staging buffers of queries and of scores both alternate.
// Arithmetic: products exact, fp32 accumulation in the matrix unit's order over all d_k coordinates (not
// per subspace first); |error| <= (d_k * 2^-24 + 2^-22) * sum_j |q_j| |c_j|, inside the bar of 1e-4 of the
// same sum that the lookup-and-sum kernel is held to.
// fp32 queries are split like the centroids (per query row, on their way into LDS); the products of the two
// small terms (2^-22 of a product) are dropped.
// Used for T >= 24, d_k in {64, 128}, d_sub a multiple of 4; everything else takes the lookup-and-sum kernel.
#include <type_traits>

#include "common.h"

namespace lookat {

typedef _Float16 pd_v8h __attribute__((ext_vector_type(8)));
typedef _Float16 pd_v4h16 __attribute__((ext_vector_type(4)));
typedef float pd_v4f __attribute__((ext_vector_type(4)));
typedef float pd_v16f __attribute__((ext_vector_type(16)));
typedef unsigned int pd_v2u __attribute__((ext_vector_type(2)));
typedef unsigned int pd_v4u __attribute__((ext_vector_type(4)));

constexpr int kPdWaves = 4;
constexpr int kPdThreads = kPdWaves * kWave;
constexpr int kPdPanel = kPdWaves * 32;        // keys per workgroup
constexpr int kPdTQ = 32;                      // queries per tile
constexpr int kPdStageStride = kPdPanel + 4;   // floats per staged score row (pad: rows 4 apart on distinct banks)
constexpr float kPdLoScale = 2048.f;

struct PrefillDenseArgs {
    const void *q;            // [BH, T, d_k] fp16 or fp32
    const float *codebooks;   // [H, m, 256, d_sub]
    const uint8_t *codes;     // (bh, l, i) at bh*code_stride + l*m + i
    float *scores;            // [BH, T, L]
    int64_t code_stride;
    int64_t L;
    int T;
    int H;
    int BH;
    int panels;               // ceil(L / 128)
    int vec4;                 // L % 4 == 0 and scores 16-byte aligned
};

// Largest |x| over the aligned group of NL consecutive lanes (NL = 16 or 32); every lane gets the result.
template <int NL>
__device__ __forceinline__ float pd_group_max(float v)
{
    v = fmaxf(v, dpp_mov<0xB1>(v, v));    // lane ^ 1
    v = fmaxf(v, dpp_mov<0x4E>(v, v));    // lane ^ 2
    v = fmaxf(v, dpp_mov<0x141>(v, v));   // the other quad of each 8
    v = fmaxf(v, dpp_mov<0x140>(v, v));   // the other 8 of each 16
    if constexpr (NL == 32) {
        float x, y;
        lanes_xor16(v, x, y);
        v = fmaxf(x, y);
    }
    return v;
}

// QT = __half: the queries are the A operand as they are.  QT = float: each query row is scaled by its own
// power of two (largest entry near 2^13) and split into two fp16 terms like the centroids, on its way into LDS;
// three products per step (hi.hi; hi.lo and lo.hi share the 2^-11 accumulator; lo.lo, 2^-22 of the product,
// is dropped) and the row's scale is undone when the tile is finished.
template <typename QT, int DK, int M>
__global__ __launch_bounds__(kPdThreads, 2) void score_prefill_dense_kernel(const PrefillDenseArgs a)
{
    constexpr bool Q32 = std::is_same<QT, float>::value;
    constexpr int DSUB = DK / M;
    constexpr int KS = DK / 16;                      // 16-coordinate steps of the contraction
    constexpr int QROW = DK * 2 + 16;                // bytes per staged query row (fp16 terms)
    constexpr int QE = 16 / (int)sizeof(QT);         // query elements per 16-byte chunk
    static_assert(DSUB % 4 == 0, "a 4-coordinate operand group lies inside one subspace");
    __shared__ __align__(16) unsigned char q_s[2][Q32 ? 2 : 1][kPdTQ * QROW];     // [buffer][hi, lo][row]
    __shared__ float qinv_s[2][kPdTQ];                                             // fp32 queries: 1 / row scale
    __shared__ __align__(16) float stage_s[2][kPdTQ * kPdStageStride];

    // workgroup ids go round-robin to the 8 dies; all panels of a (b,h) stay on one die (its queries are
    // re-read by every panel and stay in that die's L2) and run side by side there: the panels of a score
    // row are then written at about the same time, which the memory system rewards (a launch that only
    // writes -inf in this pattern: 371 us with the panels of a (b,h) side by side, 418 us with the same
    // panel of many (b,h) side by side; 4 x 32 heads x 2048 x 2048 scores)
    const int xcd = blockIdx.x % 8;
    const int slot = blockIdx.x / 8;
    const int bh = (slot / a.panels) * 8 + xcd;
    const int panel = slot % a.panels;
    if (bh >= a.BH)
        return;
    const int h = bh % a.H;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int n = lane & 31;          // key column (B operand, result), query row (A operand)
    const int g = lane >> 5;          // which half of a 16-coordinate step
    const int64_t off = a.L - a.T;    // query t sits at position t + off
    const int l0 = panel * kPdPanel;
    const QT *qg = static_cast<const QT *>(a.q) + (int64_t)bh * a.T * DK;
    float *scores_bh = a.scores + (int64_t)bh * a.T * a.L;
    const int ntiles = (a.T + kPdTQ - 1) / kPdTQ;
    // first query that sees the panel's first key, and its tile
    const int64_t t_first = (l0 - off > 0) ? (l0 - off) : 0;
    const int tile_first = (int)(t_first / kPdTQ);

    // ---- the next step's query tile: 16-byte chunks dealt to the threads, requested ahead ----
    constexpr int QCHUNKS = kPdTQ * DK * (int)sizeof(QT) / 16;          // chunks of a tile
    constexpr int CPR = DK / QE;                                        // chunks per query row
    constexpr int NQ = (QCHUNKS + kPdThreads - 1) / kPdThreads;         // chunks per thread
    static_assert(!Q32 || (QCHUNKS % kPdThreads == 0 && (CPR == 16 || CPR == 32)),
                  "fp32 queries: a row's chunks sit in 16 or 32 consecutive lanes (the row maximum is a lane-group maximum)");
    pd_v4u qreg[NQ];
#define LOOKAT_PD_FETCH_Q(tile_)                                                                          \
    _Pragma("unroll") for (int k = 0; k < NQ; ++k)                                                        \
    {                                                                                                     \
        const int c_ = tid + k * kPdThreads;              /* 16-byte chunk of the tile */                 \
        const int row_ = c_ / CPR;                                                                        \
        const int64_t t_ = (int64_t)(tile_) * kPdTQ + row_;                                               \
        qreg[k] = ((tile_) < ntiles && c_ < QCHUNKS && t_ < a.T)                                          \
                      ? *reinterpret_cast<const pd_v4u *>(qg + t_ * DK + (c_ % CPR) * QE)                 \
                      : pd_v4u{0u, 0u, 0u, 0u};                                                           \
    }
#define LOOKAT_PD_PUT_Q(buf_)                                                                             \
    _Pragma("unroll") for (int k = 0; k < NQ; ++k)                                                        \
    {                                                                                                     \
        const int c_ = tid + k * kPdThreads;                                                              \
        if constexpr (!Q32) {                                                                             \
            if (QCHUNKS % kPdThreads == 0 || c_ < QCHUNKS)                                                \
                *reinterpret_cast<pd_v4u *>(q_s[buf_][0] + (c_ / CPR) * QROW + (c_ % CPR) * 16) = qreg[k]; \
        } else {                                                                                          \
            float x_[4];                                                                                  \
            _Pragma("unroll") for (int e = 0; e < 4; ++e) x_[e] = __uint_as_float(qreg[k][e]);           \
            const float rmax_ = pd_group_max<CPR>(fmaxf(fmaxf(fabsf(x_[0]), fabsf(x_[1])), fmaxf(fabsf(x_[2]), fabsf(x_[3])))); \
            int ex_ = (int)((__float_as_uint(rmax_) >> 23) & 0xffu) - 127;                                \
            if (rmax_ == 0.f)                                                                             \
                ex_ = 0;                                                                                  \
            int se_ = 13 - ex_;                                                                           \
            se_ = se_ > 100 ? 100 : (se_ < -100 ? -100 : se_);                                            \
            const float qs_ = __uint_as_float((uint32_t)(se_ + 127) << 23);                               \
            pd_v4h16 hi_, lo_;                                                                            \
            _Pragma("unroll") for (int e = 0; e < 4; ++e)                                                 \
            {                                                                                             \
                const float w_ = qs_ * x_[e];                                                             \
                hi_[e] = (_Float16)w_;                                                                    \
                lo_[e] = (_Float16)((w_ - (float)hi_[e]) * kPdLoScale);                                   \
            }                                                                                             \
            *reinterpret_cast<pd_v4h16 *>(q_s[buf_][0] + (c_ / CPR) * QROW + (c_ % CPR) * 8) = hi_;       \
            *reinterpret_cast<pd_v4h16 *>(q_s[buf_][Q32 ? 1 : 0] + (c_ / CPR) * QROW + (c_ % CPR) * 8) = lo_; \
            if (c_ % CPR == 0)                                                                            \
                qinv_s[buf_][c_ / CPR] = __uint_as_float((uint32_t)(127 - se_) << 23);                    \
        }                                                                                                 \
    }
    LOOKAT_PD_FETCH_Q(tile_first)

    // ---- the stationary operand: centroids of this wavefront's 32 keys, by code ----
    pd_v8h b_hi[KS], b_lo[KS];
    float inv_scale;
    {
        const int64_t key = (int64_t)l0 + wave * 32 + n;
        const int64_t key_c = key < a.L ? key : a.L - 1;            // past the end: any valid key (columns not stored)
        const uint8_t *cp = a.codes + (int64_t)bh * a.code_stride + key_c * M;
        uint32_t cw[(M + 3) / 4];
        if constexpr (M == 2) {
            cw[0] = *reinterpret_cast<const uint16_t *>(cp);
        } else if constexpr (M == 4) {
            cw[0] = *reinterpret_cast<const uint32_t *>(cp);
        } else if constexpr (M == 8) {
            const pd_v2u t = *reinterpret_cast<const pd_v2u *>(cp);
            cw[0] = t.x;
            cw[1] = t.y;
        } else {
            const pd_v4u t = *reinterpret_cast<const pd_v4u *>(cp);
            cw[0] = t.x;
            cw[1] = t.y;
            cw[2] = t.z;
            cw[3] = t.w;
        }
        const float *cb_h = a.codebooks + (int64_t)h * M * kCentroids * DSUB;
        pd_v4f raw[KS][2];
        float cmax = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int dim0 = 16 * s + 8 * g + 4 * u;                  // four coordinates inside one subspace
                const int i = dim0 / DSUB;
                const uint32_t code = (cw[i / 4] >> (8 * (i % 4))) & 0xffu;
                raw[s][u] = *reinterpret_cast<const pd_v4f *>(cb_h + ((int64_t)i * kCentroids + code) * DSUB + dim0 % DSUB);
            }
        // ---- rows that cannot see any key of the panel: -inf.  Here, behind the centroid requests and ahead of
        // their use: the stores keep the memory system busy while the centroids arrive, and the wait for
        // the centroids (older in the in-order counter) does not wait for the stores ----
        {
            const int rows_masked = tile_first * kPdTQ;     // rows before the first tile that sees the panel (< T)
            const pd_v4f ninf = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            if (a.vec4) {
                // kPdPanel / 4 threads cover the panel's columns of one row; the workgroup covers 8 rows per pass
                const int c4 = tid % (kPdPanel / 4);
                if (l0 + 4 * c4 < a.L)
                    for (int r = tid / (kPdPanel / 4); r < rows_masked; r += kPdThreads / (kPdPanel / 4))
                        __builtin_nontemporal_store(ninf, reinterpret_cast<pd_v4f *>(scores_bh + (int64_t)r * a.L + l0 + 4 * c4));
            } else {
                const int c = tid & (kPdPanel - 1);
                if (l0 + c < a.L)
                    for (int r = tid / kPdPanel; r < rows_masked; r += kPdThreads / kPdPanel)
                        scores_bh[(int64_t)r * a.L + l0 + c] = -INFINITY;
            }
        }

#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                cmax = fmaxf(cmax, fabsf(raw[s][e / 4][e % 4]));
        cmax = wave_max(cmax);
        int ex = (int)((__float_as_uint(cmax) >> 23) & 0xffu) - 127;   // floor(log2(cmax)) for normal numbers
        if (cmax == 0.f)
            ex = 0;
        int se = 13 - ex;
        se = se > 100 ? 100 : (se < -100 ? -100 : se);
        const float scale = __uint_as_float((uint32_t)(se + 127) << 23);
        inv_scale = __uint_as_float((uint32_t)(127 - se) << 23);
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float w = scale * raw[s][e / 4][e % 4];         // exact: a power of two
                const _Float16 wh = (_Float16)w;
                b_hi[s][e] = wh;
                b_lo[s][e] = (_Float16)((w - (float)wh) * kPdLoScale);   // exact difference and scaling, one rounding
            }
    }

    LOOKAT_PD_PUT_Q(0)
    LOOKAT_PD_FETCH_Q(tile_first + 1)
    __syncthreads();

    // ---- query tiles that see the panel ----
    int buf = 0;
    for (int tile = tile_first; tile < ntiles; ++tile, buf ^= 1) {
        pd_v16f acc_h, acc_l;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc_h[r] = 0.f;
            acc_l[r] = 0.f;
        }
        const unsigned char *qrow = q_s[buf][0] + n * QROW + g * 16;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const pd_v8h av = *reinterpret_cast<const pd_v8h *>(qrow + s * 32);
            acc_h = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, b_hi[s], acc_h, 0, 0, 0);
            acc_l = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, b_lo[s], acc_l, 0, 0, 0);
            if constexpr (Q32) {
                const pd_v8h al = *reinterpret_cast<const pd_v8h *>(q_s[buf][1] + n * QROW + g * 16 + s * 32);
                acc_l = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, b_hi[s], acc_l, 0, 0, 0);
            }
        }
        // result register r of lane (n, g): query row 8*(r/4) + 4*g + r%4 of the tile, key column n
        const int t0 = tile * kPdTQ;
        const int64_t key = (int64_t)l0 + wave * 32 + n;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 8 * (r / 4) + 4 * g + (r % 4);
            float sc = fmaf(acc_l[r], 1.f / kPdLoScale, acc_h[r]) * inv_scale;
            if constexpr (Q32)
                sc *= qinv_s[buf][row];
            stage_s[buf][row * kPdStageStride + wave * 32 + n] = (key <= (int64_t)t0 + row + off) ? sc : -INFINITY;
        }
        LOOKAT_PD_PUT_Q(buf ^ 1)
        // One barrier per tile: the scores of this tile are staged and the next tile's queries are in LDS.
        // Both kinds of buffer alternate, so what is overwritten in the next step was last read before the
        // previous barrier.
        __syncthreads();
        // the tile after the next is requested BEFORE this tile's stores: loads and stores return through one
        // in-order counter, so the wait for these loads (a step from now) lets the stores behind them fly
        LOOKAT_PD_FETCH_Q(tile + 2)
        if (a.vec4) {
#pragma unroll
            for (int k = 0; k < (kPdTQ * kPdPanel / 4) / kPdThreads; ++k) {
                const int x = tid + k * kPdThreads;
                const int row = x / (kPdPanel / 4), c4 = x % (kPdPanel / 4);
                const pd_v4f v = *reinterpret_cast<const pd_v4f *>(stage_s[buf] + row * kPdStageStride + 4 * c4);
                if (t0 + row < a.T && l0 + 4 * c4 < a.L)
                    __builtin_nontemporal_store(v, reinterpret_cast<pd_v4f *>(scores_bh + (int64_t)(t0 + row) * a.L + l0 + 4 * c4));
            }
        } else {
#pragma unroll 4
            for (int k = 0; k < (kPdTQ * kPdPanel) / kPdThreads; ++k) {
                const int x = tid + k * kPdThreads;
                const int row = x / kPdPanel, c = x % kPdPanel;
                if (t0 + row < a.T && l0 + c < a.L)
                    scores_bh[(int64_t)(t0 + row) * a.L + l0 + c] = stage_s[buf][row * kPdStageStride + c];
            }
        }
    }
#undef LOOKAT_PD_FETCH_Q
#undef LOOKAT_PD_PUT_Q
}

template <int DK, int M>
static void launch_prefill_dense_case(const PrefillDenseArgs &a, bool q_fp32, hipStream_t st)
{
    const int64_t wgs = (int64_t)((a.BH + 7) / 8 * 8) * a.panels;
    if (q_fp32)
        hipLaunchKernelGGL((score_prefill_dense_kernel<float, DK, M>), dim3((unsigned)wgs), dim3(kPdThreads), 0, st, a);
    else
        hipLaunchKernelGGL((score_prefill_dense_kernel<__half, DK, M>), dim3((unsigned)wgs), dim3(kPdThreads), 0, st, a);
}

// d_k in {64, 128}, m in {2, 4, 8, 16}: launches and returns true; otherwise returns false and the caller
// takes the lookup-and-sum kernel.
bool launch_prefill_dense(const lookat_shape *s, int T, int64_t L, const void *q, bool q_fp32, const float *codebooks,
                          const uint8_t *codes, int64_t code_stride_bh, float *scores, hipStream_t st)
{
    PrefillDenseArgs a;
    a.q = q;
    a.codebooks = codebooks;
    a.codes = codes;
    a.scores = scores;
    a.code_stride = code_stride_bh;
    a.L = L;
    a.T = T;
    a.H = s->H;
    a.BH = s->B * s->H;
    a.panels = (int)((L + kPdPanel - 1) / kPdPanel);
    a.vec4 = (L % 4 == 0) && aligned16(scores);
    if ((int64_t)((a.BH + 7) / 8 * 8) * a.panels > 0x7fffffffLL)
        return false;
#define LOOKAT_PD_CASE(DK_, M_)                      \
    if (s->d_k == DK_ && s->m == M_) {               \
        launch_prefill_dense_case<DK_, M_>(a, q_fp32, st);   \
        return true;                                 \
    }
    LOOKAT_PD_CASE(64, 2)
    LOOKAT_PD_CASE(64, 4)
    LOOKAT_PD_CASE(64, 8)
    LOOKAT_PD_CASE(64, 16)
    LOOKAT_PD_CASE(128, 2)
    LOOKAT_PD_CASE(128, 4)
    LOOKAT_PD_CASE(128, 8)
    LOOKAT_PD_CASE(128, 16)
#undef LOOKAT_PD_CASE
    return false;
}

}  // namespace lookat
