// Causal lookup-and-sum scoring for a block of T queries (prefill): every query builds its
// lookup tables (paper Sec. 3.5, "Precomputation Lookup Tables") and scores the coded keys
// it may see (Sec. 3.5, "Lookup and Sum"; Algorithm 1, second loop), without the tables ever
// leaving the chip:
//     scores[b,h,t,l] = sum_i LUT_{b,h,t,i}[codes[b,h,l,i]]   for l <= t + (L - T),  else -inf.
//
// Shape of the computation on gfx950
//   * one workgroup (256 threads = 4 wavefronts) = one (b,h) and kPfGroup consecutive tiles of
//     TQ = 4 queries; two workgroups fit a compute unit (64 KB of tables each at m = 16), so one
//     builds tables on the matrix cores while the other gathers from LDS.  Two wavefronts per SIMD
//     leave each 256 registers: thread c keeps centroid c of EVERY subspace (d_k floats) for all
//     the workgroup's tiles, so a tile's tables cost no codebook traffic and nothing spills;
//   * the tables of a tile live in LDS as lut_s[i][c][4] (fp32): the four queries' entries of one
//     (subspace, centroid) are adjacent, so ONE 16-byte LDS read per (key, subspace) serves four
//     queries: a quarter of the gather instructions of a [query][i][c] layout;
//   * table build: per subspace the product [4 queries x d_sub] . [d_sub x 256 centroids] is done
//     with v_mfma_f32_4x4x1 (16 independent 4x4 outer products per instruction, fp32 in and out).
//     A = the four queries' coordinate j (lane%4 picks the query, the same in every block),
//     B = coordinate j of the lane's own centroid, so after d_sub instructions lane c holds the
//     four queries' entries for centroid c: exactly one 16-byte LDS store.  On the vector ALU the
//     same build costs 4 FMAs and an LDS operand read per (centroid, coordinate) and was 60% of
//     the kernel's LDS instructions;
//   * a thread scores four consecutive keys per step, so its 4 x 4 results leave as one 16-byte
//     store per query row (1 KB contiguous per wavefront and instruction);
//   * nothing is loaded from memory inside the tile loop: the workgroup's queries wait in LDS and a
//     thread's codes (the same keys for every tile) in registers.  Loads and stores share one
//     in-order counter here, so a wait for a load inside the loop would wait for the tile's 32 KB of
//     scores to drain as well;
//   * the scoring loop is bound by LDS gathers (4 bytes per (query, key, subspace)) and by the
//     scores written to HBM (4 bytes per (query, key), masked ones included).  The gathers hit
//     random bank groups: an LDS read of 16 bytes per lane is served 8 lanes at a time and 8 random
//     codes pile 2.7 deep on average (measured 21.8 cycles per gather instruction instead of 8).
//     A conflict-free variant was built and measured twice: tables as [i/8][c][i%8][4] with lane l
//     walking the subspaces in the order (u + l) % 8, and the accumulators rotated among registers
//     before the store so that 8 consecutive lanes store 8 different subspaces (either 8 accumulators
//     rotated by c%8, or odd 4-lane blocks working on subspaces 4..7,0..3 plus a rotation of 4 by
//     lane%4).  Both halve the conflict cycles; the first was 30% slower (its selects), the second
//     exactly as fast as this kernel: the gathers' bank conflicts are not what bounds it.
#include "common.h"

namespace lookat {

constexpr int kPfThreads = 256;   // = centroids per subspace: thread c owns centroid c
constexpr int kPfTQ = 4;      // queries per tile
constexpr int kPfGroup = 8;   // query tiles per workgroup (codebook registers reused) for 2-byte queries ...
template <typename QT>
constexpr int pf_group() { return sizeof(QT) == 2 ? kPfGroup : kPfGroup / 2; }   // ... half as many for fp32: the group's queries wait in LDS

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
    int groups;               // ceil(tiles / tiles per workgroup)
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

// Sum of the four queries' table entries of one key over all subspaces, ascending subspace order
// (as Algorithm 1 sums), GB gathers requested before the first is used.  Tables as [i][c][4].
template <int M>
__device__ __forceinline__ pf_v4f pf_score_key(const float *lut_s, const PfCodes<M> &kc)
{
    constexpr int GB = M < 8 ? M : 8;
    pf_v4f s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i0 = 0; i0 < M; i0 += GB) {
        pf_v4f v[GB];
#pragma unroll
        for (int u = 0; u < GB; ++u)
            v[u] = *reinterpret_cast<const pf_v4f *>(lut_s + ((i0 + u) * kCentroids + kc.byte(i0 + u)) * kPfTQ);
#pragma unroll
        for (int u = 0; u < GB; ++u)
            s += v[u];
    }
    return s;
}

// grid = 8 * ceil(BH / 8) * ceil(tiles / kPfGroup) workgroups, mapped to ((b,h), tile group) below.
template <typename QT, int DK, int M>
__global__ __launch_bounds__(kPfThreads, 2) void score_prefill_kernel(const PrefillArgs a)
{
    constexpr int TQ = kPfTQ;
    constexpr int NT = kPfThreads;
    constexpr int DSUB = DK / M;
    constexpr int QE = TQ * DK / NT;               // query elements staged per thread and tile
    constexpr int QS = DK + 4;                     // row stride of q_s in floats
    constexpr int GROUP = pf_group<QT>();
    static_assert(NT == kCentroids, "thread c owns centroid c");
    static_assert(DSUB % 4 == 0 && M % 2 == 0 && (TQ * DK) % NT == 0, "operand reads are 16 bytes wide");
    extern __shared__ __align__(16) float smem[];
    float *lut_s = smem;                           // [M][256][TQ]
    float *q_s = smem + M * kCentroids * TQ;       // [2][TQ][QS]: rows 16 bytes apart modulo the 128-byte bank row
    QT *q_all = reinterpret_cast<QT *>(q_s + 2 * TQ * QS);   // [GROUP][TQ][DK]: the queries of all the workgroup's tiles, as given
    pf_v4f *lut4 = reinterpret_cast<pf_v4f *>(lut_s);

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
    // centroid `tid` of every subspace, kept for all tiles of the workgroup
    float row[M][DSUB];
#pragma unroll
    for (int i = 0; i < M; ++i) {
        const float4 *src =
            reinterpret_cast<const float4 *>(a.codebooks + (((int64_t)h * M + i) * kCentroids + tid) * DSUB);
#pragma unroll
        for (int j4 = 0; j4 < DSUB / 4; ++j4) {
            const float4 v = src[j4];
            row[i][4 * j4] = v.x;
            row[i][4 * j4 + 1] = v.y;
            row[i][4 * j4 + 2] = v.z;
            row[i][4 * j4 + 3] = v.w;
        }
    }

    // Everything the tiles need from memory is requested here, before the first score is stored:
    // loads and stores share one in-order counter on this chip, and a wait for a load that is mixed
    // with stores waits for ALL of them, i.e. for a tile's 32 KB of scores to drain to HBM.  Inside
    // the tile loop there are then stores only.
    //   * the queries of all GROUP tiles go to LDS as they are (converted tile by tile later);
    //   * the codes a thread scores are the same for every tile (keys 4*tid .. 4*tid+3 and the
    //     same 1024 further on): two such quads stay in registers (contexts up to 2048 keys; beyond
    //     that a loop with loads takes over).  Always issued, at an index clamped into the cache:
    //     plain values, no partly written arrays.
    const int tile_lo = group * GROUP;
    const int tile_hi = (tile_lo + GROUP - 1 < a.tiles) ? tile_lo + GROUP - 1 : a.tiles - 1;
    for (int x = tid; x < GROUP * TQ * DK; x += NT) {
        const int t = tile_lo * TQ + x / DK;
        q_all[x] = (t < a.T) ? qg[(int64_t)t * DK + x % DK] : QT(0.f);
    }
    const int last_key = (int)(a.L - 1);
    PfCodes<M> ka0, ka1, ka2, ka3, kb0, kb1, kb2, kb3;
#define LOOKAT_PF_LOAD_QUAD(k0_, k1_, k2_, k3_, l0_)                                         \
    do {                                                                                     \
        const int q0_ = (l0_);                                                               \
        k0_.load(codes_bh + (int64_t)(q0_ < last_key ? q0_ : last_key) * M);                 \
        k1_.load(codes_bh + (int64_t)(q0_ + 1 < last_key ? q0_ + 1 : last_key) * M);         \
        k2_.load(codes_bh + (int64_t)(q0_ + 2 < last_key ? q0_ + 2 : last_key) * M);         \
        k3_.load(codes_bh + (int64_t)(q0_ + 3 < last_key ? q0_ + 3 : last_key) * M);         \
    } while (0)
    LOOKAT_PF_LOAD_QUAD(ka0, ka1, ka2, ka3, 4 * tid);
    LOOKAT_PF_LOAD_QUAD(kb0, kb1, kb2, kb3, 4 * tid + 4 * NT);
#define LOOKAT_PF_KEEP(k_)                                   \
    _Pragma("unroll") for (int w_ = 0; w_ < (M + 3) / 4; ++w_) asm volatile("" : "+v"(k_.w[w_]))
    // (a first "use" of the cached codes here, so that the wait for their loads sits in front of
    // the tile loop and not, re-executed with stores in flight, inside it)
    LOOKAT_PF_KEEP(ka0);
    LOOKAT_PF_KEEP(ka1);
    LOOKAT_PF_KEEP(ka2);
    LOOKAT_PF_KEEP(ka3);
    LOOKAT_PF_KEEP(kb0);
    LOOKAT_PF_KEEP(kb1);
    LOOKAT_PF_KEEP(kb2);
    LOOKAT_PF_KEEP(kb3);
    __syncthreads();   // q_all complete
    auto stage_q = [&](int tile, float *dst) {   // a tile's queries: LDS as given -> LDS fp32, padded rows
#pragma unroll
        for (int e = 0; e < QE; ++e) {
            const int x = tid + e * NT;
            dst[(x / DK) * QS + x % DK] = pf_to_f32<QT>(q_all[(tile - tile_lo) * (TQ * DK) + x]);
        }
    };
    stage_q(tile_hi, q_s);
    int cur = 0;

    for (int tile = tile_hi; tile >= tile_lo; --tile) {
        const int t0 = tile * TQ;
        const int64_t vis_last = t0 + TQ - 1 + off;                     // last key any query of the tile sees
        const int kmax = (int)((vis_last + 1 < a.L) ? vis_last + 1 : a.L);
        const float *q_lane = q_s + cur * (TQ * QS) + (tid & 3) * QS;   // matrix operand: query (lane % 4) of the tile

        __syncthreads();   // this tile's queries are staged; the previous tile's readers are done with lut_s

        // ---- tables as [i][c][4]: lut4[i*256 + c] = (q[t]^(i) . C_i[c])_{t=0..3}, j ascending ----
        // Two subspaces at a time: their accumulator chains are independent, so one chain's
        // matrix-core latency is covered by the other's instruction.
#pragma unroll
        for (int i = 0; i < M; i += 2) {
            pf_v4f acc0 = {0.f, 0.f, 0.f, 0.f};
            pf_v4f acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j4 = 0; j4 < DSUB / 4; ++j4) {
                const pf_v4f x0 = *reinterpret_cast<const pf_v4f *>(q_lane + i * DSUB + 4 * j4);
                const pf_v4f x1 = *reinterpret_cast<const pf_v4f *>(q_lane + (i + 1) * DSUB + 4 * j4);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    acc0 = __builtin_amdgcn_mfma_f32_4x4x1f32(x0[u], row[i][4 * j4 + u], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_4x4x1f32(x1[u], row[i + 1][4 * j4 + u], acc1, 0, 0, 0);
                }
            }
            lut4[i * kCentroids + tid] = acc0;
            lut4[(i + 1) * kCentroids + tid] = acc1;
        }
        if (tile > tile_lo)
            stage_q(tile - 1, q_s + (cur ^ 1) * (TQ * QS));
        cur ^= 1;
        __syncthreads();

        // ---- scoring: four consecutive keys per thread and step, four scores per key ----
        // A thread's 4 keys x 4 queries come out as four 16-byte pieces, one per query row, so a
        // wavefront writes 1 KB of contiguous scores per store instruction (with one key per lane
        // it would be 256 bytes, and the kernel's 2 GB of output four times the store instructions).
        float *rowp[TQ];   // score rows of the tile: uniform bases (scalar registers)
#pragma unroll
        for (int t = 0; t < TQ; ++t)
            rowp[t] = scores_bh + (int64_t)(t0 + t) * a.L;
        auto score_quad = [&](int l0, const PfCodes<M> &k0, const PfCodes<M> &k1, const PfCodes<M> &k2,
                              const PfCodes<M> &k3) {
            pf_v4f sc[4];
            sc[0] = pf_score_key<M>(lut_s, k0);
            sc[1] = pf_score_key<M>(lut_s, k1);
            __builtin_amdgcn_sched_barrier(0);   // two keys' gathers in flight at a time: more would only fill registers
            sc[2] = pf_score_key<M>(lut_s, k2);
            sc[3] = pf_score_key<M>(lut_s, k3);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < TQ; ++t) {
                const int tq = t0 + t;
                if (tq >= a.T)
                    continue;
                pf_v4f o;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = (l0 + j <= tq + off) ? sc[j][t] : -INFINITY;   // keys of the quad past the tile's range are masked too
                if (a.vec4) {
                    *reinterpret_cast<pf_v4f *>(rowp[t] + (uint32_t)l0) = o;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (l0 + j < a.L)
                            rowp[t][(uint32_t)(l0 + j)] = o[j];
                }
            }
        };
        // The gather addresses depend only on the cached codes, so the compiler would compute all
        // of them (8 keys x m subspaces) once, outside the tile loop, and spill them.  Declaring the
        // cached code words modified here keeps that arithmetic (a byte extract and a shift-add per
        // gather) inside the loop.
        LOOKAT_PF_KEEP(ka0);
        LOOKAT_PF_KEEP(ka1);
        LOOKAT_PF_KEEP(ka2);
        LOOKAT_PF_KEEP(ka3);
        LOOKAT_PF_KEEP(kb0);
        LOOKAT_PF_KEEP(kb1);
        LOOKAT_PF_KEEP(kb2);
        LOOKAT_PF_KEEP(kb3);
#undef LOOKAT_PF_KEEP
        if (4 * tid < kmax)
            score_quad(4 * tid, ka0, ka1, ka2, ka3);
        if (4 * tid + 4 * NT < kmax)
            score_quad(4 * tid + 4 * NT, kb0, kb1, kb2, kb3);
        for (int l0 = 4 * tid + 8 * NT; l0 < kmax; l0 += 4 * NT) {   // contexts beyond the cached quads
            PfCodes<M> kc0, kc1, kc2, kc3;
            LOOKAT_PF_LOAD_QUAD(kc0, kc1, kc2, kc3, l0);
            score_quad(l0, kc0, kc1, kc2, kc3);
        }
        // ---- keys no query of the tile may see (from the end of the last quad on) ----
        const int64_t kfill = ((int64_t)kmax + 3) / 4 * 4;
        for (int t = 0; t < TQ; ++t) {
            const int tq = t0 + t;
            if (tq >= a.T)
                break;
            if (a.vec4) {
                const pf_v4f ninf = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                for (int64_t l = kfill + 4 * tid; l < a.L; l += 4 * NT)
                    *reinterpret_cast<pf_v4f *>(rowp[t] + l) = ninf;
            } else {
                for (int64_t l = kfill + tid; l < a.L; l += NT)
                    rowp[t][l] = -INFINITY;
            }
        }
    }
}

#undef LOOKAT_PF_LOAD_QUAD

template <typename QT, int DK, int M>
static int launch_prefill(const PrefillArgs &a0, int BH, hipStream_t st)
{
    PrefillArgs a = a0;
    a.tiles = (a.T + kPfTQ - 1) / kPfTQ;
    const size_t lds = ((size_t)M * kCentroids * kPfTQ + 2 * (size_t)kPfTQ * (DK + 4)) * sizeof(float) +
                       (size_t)pf_group<QT>() * kPfTQ * DK * sizeof(QT);
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
    a.groups = (a.tiles + pf_group<QT>() - 1) / pf_group<QT>();
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
        const int64_t groups = ((int64_t)(T + kPfTQ - 1) / kPfTQ + kPfGroup / 2 - 1) / (kPfGroup / 2);   // the smaller group size
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
    a.vec4 = (L % 4 == 0) && aligned16(scores);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return (q_dtype == LOOKAT_F16) ? dispatch_prefill<__half>(shape, a, st) : dispatch_prefill<float>(shape, a, st);
}
