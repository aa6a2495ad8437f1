// Causal lookup-and-sum scoring for a block of T queries (prefill): every query builds its
// lookup tables (paper Sec. 3.5, "Precomputation Lookup Tables") and scores the coded keys
// it may see (Sec. 3.5, "Lookup and Sum"; Algorithm 1, second loop), without the tables ever
// leaving the chip:
//     scores[b,h,t,l] = sum_i LUT_{b,h,t,i}[codes[b,h,l,i]]   for l <= t + (L - T),  else -inf.
//
// Shape of the computation on gfx950
//   * queries are taken in tiles of TQ = 4; a tile's tables live in LDS as [i][c][4] (fp32): the
//     four queries' entries of one (subspace, centroid) are adjacent, so ONE 16-byte LDS read per
//     (key, subspace) serves four queries;
//   * one workgroup of 1024 threads per compute unit, two jobs on different wavefronts: wavefronts
//     0..7 build tables on the matrix cores (and fill the keys no query of a tile may see with
//     -inf), wavefronts 8..15 score.  The tables are double buffered (2 x 64 KB at m = 16), so tile
//     n is scored while tile n+1 is built: matrix-core work, vector adds and LDS gathers come from
//     different wavefronts and overlap.  (With both jobs alternating inside every wavefront, two
//     256-thread workgroups per compute unit, the phases did not overlap: time = their sum.)
//   * a workgroup stays on its (b,h) for many tiles (tiles are dealt round-robin to the workgroups
//     of a (b,h), late ones first, so all workgroups do equal work): the centroid rows and the
//     codes of the keys a thread scores are the same for every tile and are loaded once.  Nothing
//     a wavefront waits for is loaded behind its own stores: loads and stores share one in-order
//     counter, so such a wait would also wait for a tile's scores to drain to HBM.  The queries
//     of the next tiles are fetched by wavefronts that store nothing.
//   * table build: per subspace [4 queries x d_sub] . [d_sub x 256 centroids] with
//     v_mfma_f32_4x4x1 (16 independent 4x4 outer products per instruction, fp32 in and out):
//     A = the four queries' coordinate (lane%4 picks the query), B = that coordinate of the
//     lane's own centroid, so after d_sub instructions lane c holds the four queries' entries
//     for centroid c: one 16-byte LDS store;
//   * LDS serves its requests in order, and eight scoring wavefronts keep over a hundred gathers
//     queued: every LDS access of a table builder waits behind them.  So the builders touch LDS
//     as little as possible: per tile ONE batch of operand reads and the table entries.  Builder
//     wavefront w owns one half of the subspaces and 64 centroids; a thread keeps its centroid's
//     d_k/2 coordinates of that half in registers.  The queries sit in LDS permuted so that lane
//     (block kappa of its 16-lane row, query t) reads the coordinates 4r + kappa of its half with
//     a few 16-byte reads; the other three coordinates of a group of four come from the
//     neighbouring blocks of the row by DPP row rotation.  A rotation gives every block a
//     DIFFERENT coordinate of the group; the 16 blocks of the instruction are independent outer
//     products, so each thread keeps its centroid's coordinates in the matching rotated order:
//     every block still accumulates all coordinates of the subspace, in an order that depends on
//     the block (fp32 sums of d_sub terms: far inside the table tolerance);
//   * a thread scores four consecutive keys, so its 4 x 4 results leave as one 16-byte store per
//     query row (1 KB contiguous per wavefront and instruction).  The gathers of a quad run as a
//     software pipeline of groups of eight: while one group is summed the next is queued in LDS;
//   * at m = 16 the gathers (4 bytes per (query, key, subspace)) hit random bank groups — the
//     table of a subspace is [256 centroids][16 bytes] — and cost about twice a conflict-free
//     read.  A layout without conflicts (one 128-byte row per centroid holding 8 subspaces, lane
//     l gathering column (u + l) % 8, the builders rotating their entries among registers by
//     lane so that their stores spread over the columns too) was built and ran exactly as fast:
//     LDS throughput is not what bounds the kernel; vector-instruction issue (6 instructions per
//     gather, the builders' matrix and DPP instructions), dependency latency inside a wavefront
//     and the wait for the slowest wavefront at every step are.  At m <= 8 the bound is the
//     scores written to HBM (4 bytes per (query, key), masked ones included).
#include "common.h"

namespace lookat {

constexpr int kPfThreads = 256;   // = centroids per subspace
constexpr int kPfTQ = 4;          // queries per tile

typedef unsigned int pf_v4u __attribute__((ext_vector_type(4)));
typedef unsigned int pf_v2u __attribute__((ext_vector_type(2)));
typedef float pf_v4f __attribute__((ext_vector_type(4)));

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
    int groups;               // workgroups per (b,h)
    int vec4;                 // L % 4 == 0 and scores 16-byte aligned: rows take 16-byte stores
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

constexpr int kPfBuildThreads = 2 * kPfThreads;               // eight table-building wavefronts
constexpr int kPfScoreThreads = 2 * kPfThreads;               // eight scoring wavefronts: 2048 keys, one quad per thread
constexpr int kPfWgThreads = kPfBuildThreads + kPfScoreThreads;

// DPP row_ror:n (rotate right within a 16-lane row): lane l receives the value of lane (l - n) % 16,
// so rotation 4k brings block kappa the operand of block (kappa - k) % 4.
template <int N>
__device__ __forceinline__ float pf_row_from(float x)
{
    if constexpr (N == 0)
        return x;
    else   // every lane is written, so there is no previous value to keep (and no copy to make first)
        return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x120 + N, 0xf, 0xf, false));
}

// LDS byte offset of the table of subspace i in buffer b (4 KB each: [256 centroids][4 queries] fp32).
// The two buffers of a subspace are neighbours, so that one address register per gather serves both
// with a compile-time offset.
__host__ __device__ constexpr uint32_t pf_slot(int i, int b) { return (uint32_t)(((i % 8) * 2 + b) * 4096 + (i / 8) * 65536); }
__host__ __device__ constexpr size_t pf_table_bytes(int m) { return m <= 8 ? (size_t)m * 8192 : 131072; }

// Workgroups per (b,h).  A workgroup fills a compute unit and all workgroups of a launch do the same
// work, so the launch proceeds in rounds of 256: the smallest count whose last round is at least 95%
// full (else the fullest), leaving every workgroup eight tiles or more to spread its set-up over.
static int pf_workgroups(int BH, int tiles)
{
    const int jmax = tiles >= 16 ? (tiles / 8 < 64 ? tiles / 8 : 64) : 1;
    int best = 1;
    double best_eff = 0.0;
    for (int j = 1; j <= jmax; ++j) {
        const double wg = (double)BH * j;
        const double rounds = (double)((BH * (long long)j + 255) / 256);
        const double eff = wg / (rounds * 256.0);
        if (eff > best_eff + 1e-9) {
            best_eff = eff;
            best = j;
        }
        if (eff >= 0.95)
            return j;
    }
    return best;
}

typedef const __attribute__((address_space(3))) pf_v4f *PfLdsEntry;
typedef __attribute__((address_space(3))) pf_v4f *PfLdsStore;

// Scores of four keys against the tile's four queries from table buffer BUF: per key the sum over the
// subspaces, ascending (as Algorithm 1 sums), of the 16-byte entries [4 queries].  The gathers run as
// a software pipeline of groups of up to 8: while one group is summed the next is already queued in
// LDS, so the wavefront always has requests in flight (summing a whole key before requesting the
// next left LDS idle while the adds ran, and the adds idle while LDS worked: the two times added up).
template <int M, int BUF>
__device__ __forceinline__ void pf_score_quad_buf(uint32_t lds_base, const PfCodes<M> (&kq)[4], pf_v4f (&sc)[4])
{
    constexpr int GS = M < 8 ? M : 8;   // gathers per group
    constexpr int GPK = M / GS;         // groups per key
    constexpr int NG = 4 * GPK;
    pf_v4f land[2][GS];
#define LOOKAT_PF_ISSUE(g_)                                                                              \
    _Pragma("unroll") for (int u = 0; u < GS; ++u)                                                       \
        land[(g_) & 1][u] = *reinterpret_cast<PfLdsEntry>(                                               \
            lds_base + kq[(g_) / GPK].byte(((g_) % GPK) * GS + u) * 16u + pf_slot(((g_) % GPK) * GS + u, BUF));
    LOOKAT_PF_ISSUE(0)
    LOOKAT_PF_ISSUE(1)
    __builtin_amdgcn_sched_barrier(0);
    pf_v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < NG; ++g) {
#pragma unroll
        for (int u = 0; u < GS; ++u)
            acc = (g % GPK == 0 && u == 0) ? land[g & 1][u] : acc + land[g & 1][u];
        if (g % GPK == GPK - 1)
            sc[g / GPK] = acc;
        if (g + 2 < NG) {
            LOOKAT_PF_ISSUE(g + 2)
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#undef LOOKAT_PF_ISSUE
}

template <typename QT, int DK, int M>
__global__ __launch_bounds__(kPfWgThreads, 1) void score_prefill_kernel(const PrefillArgs a)
{
    constexpr int TQ = kPfTQ;
    constexpr int NB = kPfBuildThreads;            // table-building threads
    constexpr int NF = NB / 2;                     // ... of which the first half also fills, the second half fetches queries
    constexpr int NS = kPfScoreThreads;            // scoring threads
    constexpr int DSUB = DK / M;
    constexpr int HALF = DK / 2;                   // coordinates per builder half
    constexpr int R = HALF / 4;                    // operand values a builder lane holds per tile
    constexpr int PAIR = (M >= 4) ? 2 : 1;         // subspaces built together
    constexpr int QSLOT = 2 * TQ * 4 * R;          // floats of one tile's permuted queries (= TQ * DK)
    constexpr int QE = TQ * DK / NF;               // query elements a fetching thread moves per tile
    static_assert(DSUB % 4 == 0 && M % 2 == 0 && R % 4 == 0 && (TQ * DK) % NF == 0, "operand reads are 16 bytes wide");
    extern __shared__ __align__(16) float smem[];
    float *q_p = smem + pf_table_bytes(M) / sizeof(float);   // [2 slots][2 halves][TQ][4 blocks][R] fp32, permuted
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float *)smem;

    // a.groups workgroups per (b,h); workgroup j of them takes the tiles tiles-1-j, tiles-1-j-groups, ...
    // (late tiles see more keys: dealing them round-robin gives every workgroup the same work).
    // Workgroup ids go round-robin to the 8 dies; a die only sees the heads congruent to its index.
    const int xcd = blockIdx.x % 8;
    const int slot = blockIdx.x / 8;
    const int bh_per_xcd = (a.BH + 7) / 8;
    const int bh = (slot % bh_per_xcd) * 8 + xcd;
    const int j_wg = slot / bh_per_xcd;
    if (bh >= a.BH || a.tiles - 1 - j_wg < 0)
        return;
    const int h = bh % a.H;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
    const bool builds = wave < NB / kWave;
    const int tid = builds ? (int)threadIdx.x : (int)threadIdx.x - NB;   // index within the role
    const int64_t off = a.L - a.T;
    const QT *qg = static_cast<const QT *>(a.q) + (int64_t)bh * a.T * DK;
    const uint8_t *codes_bh = a.codes + (int64_t)bh * a.code_stride;
    float *scores_bh = a.scores + (int64_t)bh * a.T * a.L;
    const int tile_first = a.tiles - 1 - j_wg;
    const int stride = a.groups;
    const int n = tile_first / stride + 1;        // tiles of this workgroup: tile_first - k*stride, k = 0 .. n-1
    // Step s = 0 .. n: tile k = s is built into table buffer s % 2 while tile k = s-1 is scored from the
    // other one; one workgroup barrier per step (both roles run the same count).

    if (builds) {
        const int half = (wave / 2) & 1;                 // subspaces half*M/2 .. +M/2-1 (wavefronts 0,1,4,5 / 2,3,6,7)
        const bool fetches = wave >= NF / kWave;         // wavefronts 4..7 move the queries, 0..3 fill
        const int c = (wave & 1) * 64 + ((wave >> 2) & 1) * 128 + (tid & 63);   // the thread's centroid
        const int kappa = (tid >> 2) & 3;                // its 4-lane block within the 16-lane row
        const int ft = tid & (NF - 1);                   // index among the filling / fetching threads
        // the centroid's coordinates of this half; register 4r+k holds coordinate 4r + (kappa - k) % 4,
        // the one that rotation 4k brings to this block
        float row[HALF];
#pragma unroll
        for (int il = 0; il < M / 2; ++il) {
            const float *src = a.codebooks + (((int64_t)h * M + half * (M / 2) + il) * kCentroids + c) * DSUB;
#pragma unroll
            for (int j4 = 0; j4 < DSUB / 4; ++j4) {
                const float4 v = *reinterpret_cast<const float4 *>(src + 4 * j4);
                const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int w = (kappa - k) & 3;
                    row[il * DSUB + 4 * j4 + k] = (w == 0) ? e[0] : (w == 1) ? e[1] : (w == 2) ? e[2] : e[3];
                }
            }
        }
        // A tile's queries travel global memory -> registers of the fetching wavefronts (one step
        // ahead) -> LDS, permuted: q_p[slot][half][t][kappa][r] = q[tile, query t][half*HALF + 4r + kappa]
        // (one more step ahead) -> operand registers of all builders (one more step).  The fetching
        // wavefronts issue no stores, so waiting for their loads does not wait for anybody's scores.
        QT qf[QE], qf0[QE], qf1[QE];
#define LOOKAT_PF_FETCH_Q(k_, dst_)                                                                      \
    _Pragma("unroll") for (int e = 0; e < QE; ++e)                                                       \
    {                                                                                                    \
        const int x_ = ft + e * NF;                                                                      \
        const int64_t t_ = (int64_t)(tile_first - (k_) * stride) * TQ + x_ / DK;                         \
        dst_[e] = ((k_) < n && t_ < a.T) ? qg[t_ * DK + x_ % DK] : QT(0.f);                              \
    }
#define LOOKAT_PF_PUT_Q(slot_, src_)                                                                     \
    _Pragma("unroll") for (int e = 0; e < QE; ++e)                                                       \
    {                                                                                                    \
        const int x_ = ft + e * NF;                                                                      \
        const int tq_ = x_ / DK, jh_ = (x_ % DK) / HALF, jl_ = (x_ % DK) % HALF;                         \
        q_p[(slot_) * QSLOT + ((jh_ * TQ + tq_) * 4 + (jl_ & 3)) * R + (jl_ >> 2)] = pf_to_f32<QT>(src_[e]); \
    }
        const float *q_lane = q_p + ((half * TQ + (tid & 3)) * 4 + kappa) * R;
        pf_v4f qv[R / 4];
#define LOOKAT_PF_LOAD_OPERAND(slot_)                                                                    \
    _Pragma("unroll") for (int r4 = 0; r4 < R / 4; ++r4)                                                 \
        qv[r4] = *reinterpret_cast<const pf_v4f *>(q_lane + (slot_) * QSLOT + 4 * r4);
        if (fetches) {
            LOOKAT_PF_FETCH_Q(0, qf0)
            LOOKAT_PF_FETCH_Q(1, qf1)
            LOOKAT_PF_FETCH_Q(2, qf)
            LOOKAT_PF_PUT_Q(0, qf0)
            LOOKAT_PF_PUT_Q(1, qf1)
        }
        uint32_t st_lo = lds_base + (uint32_t)c * 16u;   // table entries of centroid c: two bases, a ds_write offset spans 64 KB
        uint32_t st_hi = st_lo + 65536u;
        asm volatile("" : "+v"(st_lo), "+v"(st_hi));
        __syncthreads();   // the first two tiles' queries are in LDS
        LOOKAT_PF_LOAD_OPERAND(0)
        __syncthreads();
#define LOOKAT_PF_BUILD_STEP(BUF_, s_)                                                                   \
    if ((s_) < n) {                                                                                      \
        const int tile_ = tile_first - (s_) * stride;                                                    \
        /* PAIR subspaces at a time: their accumulator chains are independent, so one chain's */        \
        /* matrix-core latency is covered by the other's instruction */                                  \
        _Pragma("unroll") for (int il = 0; il < M / 2; il += PAIR)                                       \
        {                                                                                                \
            pf_v4f acc[PAIR];                                                                            \
            _Pragma("unroll") for (int p = 0; p < PAIR; ++p) acc[p] = pf_v4f{0.f, 0.f, 0.f, 0.f};        \
            _Pragma("unroll") for (int j4 = 0; j4 < DSUB / 4; ++j4)                                      \
            {                                                                                            \
                float x[PAIR];                                                                           \
                _Pragma("unroll") for (int p = 0; p < PAIR; ++p)                                         \
                    x[p] = qv[(((il + p) * DSUB) / 4 + j4) / 4][(((il + p) * DSUB) / 4 + j4) % 4];       \
                _Pragma("unroll") for (int p = 0; p < PAIR; ++p)                                         \
                    acc[p] = __builtin_amdgcn_mfma_f32_4x4x1f32(pf_row_from<0>(x[p]), row[(il + p) * DSUB + 4 * j4 + 0], acc[p], 0, 0, 0);  \
                _Pragma("unroll") for (int p = 0; p < PAIR; ++p)                                         \
                    acc[p] = __builtin_amdgcn_mfma_f32_4x4x1f32(pf_row_from<4>(x[p]), row[(il + p) * DSUB + 4 * j4 + 1], acc[p], 0, 0, 0);  \
                _Pragma("unroll") for (int p = 0; p < PAIR; ++p)                                         \
                    acc[p] = __builtin_amdgcn_mfma_f32_4x4x1f32(pf_row_from<8>(x[p]), row[(il + p) * DSUB + 4 * j4 + 2], acc[p], 0, 0, 0);  \
                _Pragma("unroll") for (int p = 0; p < PAIR; ++p)                                         \
                    acc[p] = __builtin_amdgcn_mfma_f32_4x4x1f32(pf_row_from<12>(x[p]), row[(il + p) * DSUB + 4 * j4 + 3], acc[p], 0, 0, 0); \
            }                                                                                            \
            _Pragma("unroll") for (int p = 0; p < PAIR; ++p)                                             \
            {                                                                                            \
                if (half == 0)                                                                           \
                    *reinterpret_cast<PfLdsStore>((il + p < 8 ? st_lo : st_hi) + (pf_slot(il + p, BUF_) & 0xffffu)) = acc[p];                  \
                else                                                                                     \
                    *reinterpret_cast<PfLdsStore>((M / 2 + il + p < 8 ? st_lo : st_hi) + (pf_slot(M / 2 + il + p, BUF_) & 0xffffu)) = acc[p];  \
            }                                                                                            \
        }                                                                                                \
        if (fetches) {                                                                                   \
            /* tile s+2 (fetched during the last step) to the LDS slot tile s has left; tile s+3 requested */ \
            LOOKAT_PF_PUT_Q(BUF_, qf)                                                                    \
            LOOKAT_PF_FETCH_Q((s_) + 3, qf)                                                              \
        } else {                                                                                         \
            /* keys no query of the tile may see */                                                      \
            const int t0_ = tile_ * TQ;                                                                  \
            const int64_t vis_ = t0_ + TQ - 1 + off;                                                     \
            const int64_t kmax_ = (vis_ + 1 < a.L) ? vis_ + 1 : a.L;                                     \
            const int64_t kfill_ = (kmax_ + 3) / 4 * 4;                                                  \
            for (int t = 0; t < TQ && t0_ + t < a.T; ++t) {                                              \
                float *rowp_ = scores_bh + (int64_t)(t0_ + t) * a.L;                                     \
                if (a.vec4) {                                                                            \
                    const pf_v4f ninf = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};                    \
                    for (uint32_t l = (uint32_t)kfill_ + 4 * ft; l < (uint32_t)a.L; l += 4 * NF)         \
                        __builtin_nontemporal_store(ninf, reinterpret_cast<pf_v4f *>(rowp_ + l));        \
                } else {                                                                                 \
                    for (uint32_t l = (uint32_t)kfill_ + ft; l < (uint32_t)a.L; l += NF)                 \
                        rowp_[l] = -INFINITY;                                                            \
                }                                                                                        \
            }                                                                                            \
        }                                                                                                \
        LOOKAT_PF_LOAD_OPERAND((BUF_) ^ 1)   /* tile s+1, in LDS since the last step */                  \
    }
        for (int s = 0; s <= n; s += 2) {
            LOOKAT_PF_BUILD_STEP(0, s)
            __syncthreads();
            LOOKAT_PF_BUILD_STEP(1, s + 1)
            __syncthreads();
        }
#undef LOOKAT_PF_BUILD_STEP
#undef LOOKAT_PF_LOAD_OPERAND
#undef LOOKAT_PF_PUT_Q
#undef LOOKAT_PF_FETCH_Q
    } else {
        // A thread scores the same four consecutive keys (4*tid ..) in every tile, so their codes stay in
        // registers (contexts up to 2048 keys; beyond that a loop with loads takes over).
        const int last_key = (int)(a.L - 1);
        const int l_own = 4 * tid;
        PfCodes<M> kq[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            kq[k].load(codes_bh + (int64_t)(l_own + k < last_key ? l_own + k : last_key) * M);
#define LOOKAT_PF_KEEP_CODES(k_)                                                                         \
    _Pragma("unroll") for (int w_ = 0; w_ < (M + 3) / 4; ++w_) asm volatile("" : "+v"(k_.w[w_]));
        LOOKAT_PF_KEEP_CODES(kq[0])
        LOOKAT_PF_KEEP_CODES(kq[1])
        LOOKAT_PF_KEEP_CODES(kq[2])
        LOOKAT_PF_KEEP_CODES(kq[3])
        __syncthreads();
        __syncthreads();
#define LOOKAT_PF_STORE_QUAD(l0_, sc_)                                                                   \
    _Pragma("unroll") for (int t = 0; t < TQ; ++t)                                                       \
    {                                                                                                    \
        const int tq_ = t0_ + t;                                                                         \
        if (tq_ < a.T) {                                                                                 \
            float *rowp_ = scores_bh + (int64_t)tq_ * a.L;                                               \
            pf_v4f o_;                                                                                   \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                \
                o_[j] = ((l0_) + j <= tq_ + (int)off) ? sc_[j][t] : -INFINITY;                           \
            if (a.vec4) {                                                                                \
                __builtin_nontemporal_store(o_, reinterpret_cast<pf_v4f *>(rowp_ + (uint32_t)(l0_)));    \
            } else {                                                                                     \
                _Pragma("unroll") for (int j = 0; j < 4; ++j)                                            \
                    if ((l0_) + j < a.L)                                                                 \
                        rowp_[(uint32_t)((l0_) + j)] = o_[j];                                            \
            }                                                                                            \
        }                                                                                                \
    }
#define LOOKAT_PF_SCORE_QUAD(BUF_, l0_, kq_)                                                             \
    {                                                                                                    \
        pf_v4f sc_[4];                                                                                   \
        pf_score_quad_buf<M, BUF_>(lds_base, kq_, sc_);                                                  \
        LOOKAT_PF_STORE_QUAD(l0_, sc_)                                                                   \
    }
#define LOOKAT_PF_SCORE_STEP(BUF_, s_)                                                                   \
    if ((s_) >= 1 && (s_) <= n) {                                                                        \
        const int t0_ = (tile_first - ((s_) - 1) * stride) * TQ;                                         \
        const int64_t vis_ = t0_ + TQ - 1 + off;                                                         \
        const int kmax_ = (int)((vis_ + 1 < a.L) ? vis_ + 1 : a.L);                                      \
        /* the address arithmetic of the cached codes stays here, inside the loop: hoisted out, the */   \
        /* addresses of all (key, subspace) pairs would want 64 more registers */                        \
        LOOKAT_PF_KEEP_CODES(kq[0])                                                                      \
        LOOKAT_PF_KEEP_CODES(kq[1])                                                                      \
        LOOKAT_PF_KEEP_CODES(kq[2])                                                                      \
        LOOKAT_PF_KEEP_CODES(kq[3])                                                                      \
        if (l_own < kmax_)                                                                               \
            LOOKAT_PF_SCORE_QUAD(BUF_, l_own, kq)                                                        \
        for (int l0 = l_own + 4 * NS; l0 < kmax_; l0 += 4 * NS) {                                        \
            PfCodes<M> kc_[4];                                                                           \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                \
                kc_[j].load(codes_bh + (int64_t)(l0 + j < last_key ? l0 + j : last_key) * M);            \
            LOOKAT_PF_SCORE_QUAD(BUF_, l0, kc_)                                                          \
        }                                                                                                \
    }
        for (int s = 0; s <= n; s += 2) {
            LOOKAT_PF_SCORE_STEP(1, s)        // tile s-1 sits in buffer (s-1) % 2 = 1
            __syncthreads();
            LOOKAT_PF_SCORE_STEP(0, s + 1)
            __syncthreads();
        }
#undef LOOKAT_PF_SCORE_STEP
#undef LOOKAT_PF_SCORE_QUAD
#undef LOOKAT_PF_STORE_QUAD
#undef LOOKAT_PF_KEEP_CODES
    }
}

template <typename QT, int DK, int M>
static int launch_prefill(const PrefillArgs &a0, int BH, hipStream_t st)
{
    PrefillArgs a = a0;
    a.tiles = (a.T + kPfTQ - 1) / kPfTQ;
    a.BH = BH;
    a.groups = pf_workgroups(BH, a.tiles);
    const size_t lds = pf_table_bytes(M) + 2 * (size_t)kPfTQ * DK * sizeof(float);   // two table buffers, two tiles of queries
    auto kern = score_prefill_kernel<QT, DK, M>;
    if (lds > 64 * 1024) {
        // allow more than 64 KB of dynamic LDS: idempotent, so every call makes it (no flag shared between host threads)
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return fail(LOOKAT_ERR_HIP, "lookat_score_prefill: cannot reserve %zu bytes of LDS: %s", lds,
                        hipGetErrorString(e));
    }
    dim3 grid((unsigned)((BH + 7) / 8 * 8 * a.groups));
    hipLaunchKernelGGL(kern, grid, dim3(kPfWgThreads), lds, st, a);
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

// prefill_dense.hip: the same scores as a dense contraction against the keys' centroids on the matrix cores
// (d_k in {64, 128}, m in {2, 4, 8, 16}); returns false when it does not take the shape.
bool launch_prefill_dense(const lookat_shape *s, int T, int64_t L, const void *q, bool q_fp32, const float *codebooks,
                          const uint8_t *codes, int64_t code_stride_bh, float *scores, hipStream_t st);

// From this many queries per (b,h) on, blocks of queries are scored on the matrix cores.  Its workgroups
// spend their first microseconds fetching centroids, which a short block does not repay: measured at 4 x 32
// heads, 4096 keys, d_k 128, m 16 (us per call, matrix cores / lookup-and-sum): T = 8: 40 / 22, 16: 40 / 34,
// 24: 40 / 46, 32: 41 / 57, 64: 52 / 67, 256: 135 / 236.
constexpr int kPfDenseMinT = 24;

static int score_prefill_impl(const lookat_shape *shape, int32_t T, int64_t L, const void *q, lookat_dtype q_dtype,
                              const float *codebooks, const uint8_t *codes, int64_t code_stride_bh,
                              float *scores, void *stream, bool allow_dense)
{
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (T <= 0 || L < T)
        return fail(LOOKAT_ERR_SHAPE, "need 1 <= T <= L (T=%d, L=%lld)", T, (long long)L);
    if (q_dtype != LOOKAT_F16 && q_dtype != LOOKAT_F32)
        return fail(LOOKAT_ERR_DTYPE, "q_dtype=%d is neither LOOKAT_F16 nor LOOKAT_F32", q_dtype);
    if (!q || !codebooks || !codes || !scores)
        return fail(LOOKAT_ERR_NULL, "q, codebooks, codes and scores must be non-NULL");
    if (L > (1LL << 30))
        return fail(LOOKAT_ERR_UNSUPPORTED, "L=%lld: a row of scores is addressed with 32-bit byte offsets (L <= 2^30)", (long long)L);
    if (code_stride_bh < L * shape->m)
        return fail(LOOKAT_ERR_SHAPE, "code_stride_bh=%lld is smaller than L*m", (long long)code_stride_bh);
    if (!aligned16(q) || !aligned16(codebooks) || (reinterpret_cast<uintptr_t>(scores) & 3u))
        return fail(LOOKAT_ERR_ALIGN, "q and codebooks must be 16-byte aligned, scores 4-byte aligned");
    const int cvec = (shape->m == 2 || shape->m == 4 || shape->m == 8 || shape->m == 16) ? shape->m : 1;
    if ((reinterpret_cast<uintptr_t>(codes) % cvec) || (code_stride_bh % cvec))
        return fail(LOOKAT_ERR_ALIGN, "codes and code_stride_bh must be multiples of %d bytes for m=%d", cvec, shape->m);
    if (((int64_t)shape->B * shape->H + 7) / 8 * 8 * 64 > 0x7fffffffLL)   // at most 64 workgroups per (b,h)
        return fail(LOOKAT_ERR_UNSUPPORTED, "B*H=%lld exceeds one launch", (long long)shape->B * shape->H);
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
    a.vec4 = (L % 4 == 0) && aligned16(scores);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (allow_dense && T >= kPfDenseMinT &&
        launch_prefill_dense(shape, T, L, q, q_dtype == LOOKAT_F32, codebooks, codes, code_stride_bh, scores, st))
        return check_launch("lookat_score_prefill");
    return (q_dtype == LOOKAT_F16) ? dispatch_prefill<__half>(shape, a, st) : dispatch_prefill<float>(shape, a, st);
}

}  // namespace lookat

extern "C" int lookat_score_prefill(const lookat_shape *shape, int32_t T, int64_t L, const void *q, lookat_dtype q_dtype,
                                    const float *codebooks, const uint8_t *codes, int64_t code_stride_bh,
                                    float *scores, void *stream)
{
    return lookat::score_prefill_impl(shape, T, L, q, q_dtype, codebooks, codes, code_stride_bh, scores, stream, true);
}

extern "C" int lookat_probe_score_prefill_lookup(const lookat_shape *shape, int32_t T, int64_t L, const void *q,
                                                 lookat_dtype q_dtype, const float *codebooks, const uint8_t *codes,
                                                 int64_t code_stride_bh, float *scores, void *stream)
{
    return lookat::score_prefill_impl(shape, T, L, q, q_dtype, codebooks, codes, code_stride_bh, scores, stream, false);
}
