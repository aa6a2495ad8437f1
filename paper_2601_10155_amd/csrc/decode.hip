// Attention decode over the product-quantised key cache (paper Algorithm 1 after the
// table build): s_l = sum_i LUT_i[code_l[i]] (Sec. 3.5 "Lookup and Sum"), softmax of
// scale*s, weighted sum of the fp16 values.
//
// Shape of the computation on gfx950
//   * the value stream (2*d_k bytes per key) and the code stream (m bytes per key) are
//     each read exactly once with 16-byte-per-lane loads, a wavefront covering 1 KB of
//     contiguous memory per load instruction;
//   * the table of one (b,h) (m KB) is staged in LDS once per workgroup and gathered
//     with one ds_read_b32 per (key, subspace);
//   * every wavefront owns 64-key tiles and keeps its own running max / sum / output
//     (online softmax), so the streaming loop has no workgroup barrier;
//   * the sequence is cut into `splits` ranges per (b,h) (flash-decoding style); the
//     ranges are merged by a second small kernel.
#include <mutex>
#include <type_traits>

#include "decode_common.h"
#include "lookat_probe.h"

namespace lookat {

struct DecodeArgs {
    const float *lut;        // [BH, m, 256]
    const uint8_t *codes;    // (bh, l, i) at bh*code_stride + l*m + i
    const __half *values;    // (bh, l, j) at bh*value_stride + l*d_k + j
    float *part;             // [BH, splits, d_k + 2]   (o[d_k], max, sum), unused when splits == 1
    float *out;              // [BH, d_k]
    float *scores_out;       // [BH, L] or nullptr
    int64_t code_stride;
    int64_t value_stride;
    int64_t L;
    int64_t keys_per_split;  // multiple of kTile
    int BH;
    int splits;
    int d_k;
    int m;
    float scale_log2e;       // scale * log2(e): the softmax runs in base 2
    // fused decode step only (lookat_decode_step): the table is built and the new key encoded in-kernel
    const void *q;           // [BH, d_k]
    const void *k_new;       // [BH, d_k]
    const float *codebooks;  // [H, m, 256, d_sub]
    uint8_t *codes_w;        // same cache as `codes`, writable: row L-1 receives the new key's codes
    int H;
};

// Kernel parameters.  The first 14 dwords of a kernel's arguments are delivered in scalar
// registers at wave launch (kernarg preload, -amdgpu-kernarg-preload-count); anything after
// them costs a round trip to memory before it can be used (about a microsecond on a fresh
// argument block, and a 52 MB decode launch lasts about ten).  So everything a wavefront needs
// before it can request its first tile travels in those 14 dwords, as scalars, and the rest
// follows in a struct that is read while the tile is in flight.
struct DecodeLate {
    float *part;
    float *out;
    float *scores_out;
    const void *q;
    const void *k_new;
    uint8_t *codes_w;
    int d_k;
    int m;
};
#define LOOKAT_DECODE_HEAD_PARAMS                                                                              \
    int p_BH, int p_splits, int p_H, const void *p_table, const uint8_t *p_codes, const __half *p_values,     \
        uint32_t p_code_stride, uint32_t p_value_stride, uint32_t p_L, uint32_t p_kps, float p_scale_log2e
#define LOOKAT_DECODE_HEAD_ARGS(a, fused)                                                                      \
    (a).BH, (a).splits, (a).H, ((fused) ? static_cast<const void *>((a).codebooks) : static_cast<const void *>((a).lut)), \
        (a).codes, (a).values, (uint32_t)(a).code_stride, (uint32_t)(a).value_stride, (uint32_t)(a).L,        \
        (uint32_t)(a).keys_per_split, (a).scale_log2e
static DecodeLate late_of(const DecodeArgs &a)
{
    return DecodeLate{a.part, a.out, a.scores_out, a.q, a.k_new, a.codes_w, a.d_k, a.m};
}
__device__ __forceinline__ DecodeArgs rebuild_args(LOOKAT_DECODE_HEAD_PARAMS, const DecodeLate &late, bool fused)
{
    DecodeArgs a;
    a.lut = fused ? nullptr : static_cast<const float *>(p_table);
    a.codebooks = fused ? static_cast<const float *>(p_table) : nullptr;
    a.codes = p_codes;
    a.values = p_values;
    a.part = late.part;
    a.out = late.out;
    a.scores_out = late.scores_out;
    a.code_stride = p_code_stride;
    a.value_stride = p_value_stride;
    a.L = p_L;
    a.keys_per_split = p_kps;
    a.BH = p_BH;
    a.splits = p_splits;
    a.d_k = late.d_k;
    a.m = late.m;
    a.scale_log2e = p_scale_log2e;
    a.q = late.q;
    a.k_new = late.k_new;
    a.codes_w = late.codes_w;
    a.H = p_H;
    return a;
}

// Workgroup id -> (bh, split).  Consecutive workgroup ids land on different dies, each
// with its own L2; this mapping keeps all splits of one (b,h) on one die so that its
// table is fetched into a single L2.
__device__ __forceinline__ bool map_block_n(const DecodeArgs &a, int count, int &unit, int &split)
{
    const int bid = blockIdx.x;
    const int xcd = bid % kXcds;
    const int slot = bid / kXcds;
    unit = (slot / a.splits) * kXcds + xcd;
    split = slot % a.splits;
    return unit < count;
}
__device__ __forceinline__ bool map_block(const DecodeArgs &a, int &bh, int &split)
{
    return map_block_n(a, a.BH, bh, split);
}

// LDS of one batch entry of the fused step (table, per-wavefront partial results, the encoder's per-wavefront
// minima and indices), rounded to 16 bytes: the distance between the two entries' blocks of a paired workgroup.
__host__ __device__ constexpr size_t step_pair_lds_bytes(int m, int d_k)
{
    return ((((size_t)m * kCentroids + (size_t)(2 * kDecWaves) * (d_k + 2)) * sizeof(float) +
             (size_t)m * kDecWaves * (sizeof(double) + sizeof(int))) + 15) / 16 * 16;
}

// ---- pieces of the fused decode step ---------------------------------------------------
template <typename T>
__device__ __forceinline__ float step_f32(T v);
template <>
__device__ __forceinline__ float step_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float step_f32<__half>(__half v) { return __half2float(v); }

// Squared distance of the encoder (paper Sec. 3.4 "Encoding"), exactly as lookat_encode_keys
// evaluates it: fp64, ascending coordinates, one rounding per subtract, multiply and add.
// A dense, 16-byte aligned, read-only array of T addressed uniformly over the wavefront, read
// as 32-bit words through the constant address space: the compiler turns these into scalar
// loads (an s_load needs dword alignment, which a __half pointer would not promise).
typedef const __attribute__((address_space(4))) uint32_t *UniformWords;
template <typename T>
__device__ __forceinline__ float uniform_elem(UniformWords p, int idx);
template <>
__device__ __forceinline__ float uniform_elem<float>(UniformWords p, int idx)
{
    return __uint_as_float(p[idx]);
}
template <>
__device__ __forceinline__ float uniform_elem<__half>(UniformWords p, int idx)
{
    const uint32_t w = p[idx >> 1];
    return __half2float(__ushort_as_half((unsigned short)((idx & 1) ? (w >> 16) : (w & 0xffffu))));
}

template <typename KT, int DSUB>
__device__ __forceinline__ double step_sq_dist(UniformWords x, int x0, const float (&y)[DSUB])
{
#pragma clang fp contract(off)
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < DSUB; ++j) {
        double diff = (double)uniform_elem<KT>(x, x0 + j) - (double)y[j];
        double sq = diff * diff;
        acc = acc + sq;
    }
    return acc;
}

// One 64-key tile of a wavefront: its codes (kc) and first CH value-row groups (v) are in
// registers or in flight.  Scores one key per lane (key = kb + kofs), updates the running
// max / sum, and accumulates the weighted value rows.
//
// MM (grouped queries, d_k = 128, G >= 4): the weighted value sum of the tile is a dense contraction
// [G query heads x 64 keys] . [64 keys x 128 coordinates] and runs on the matrix cores
// (v_mfma_f32_16x16x16_f16, fp32 accumulate) instead of G x 128 multiply-adds per key on the vector ALU:
//   * A operand = value rows, as loaded: lane (rowin, sub) holds 8 coordinates of the rows 4j + rowin of a
//     16-key step, j = 0..3.  With the instruction's contraction index k = 4*rowin + j standing for key
//     4j + rowin, the four halves a lane must supply for coordinate 8*sub + e are element e of its four
//     loads: two byte permutes per instruction, no data crosses lanes.  Instruction e of a step handles the
//     coordinates {8*s + e}: row s of its 16 x 16 result is coordinate 8*s + e;
//   * B operand = weights: column n < G is the weight of query head n rounded to fp16, column G + n the
//     remainder (p - fp16(p)) * 2^11 rounded to fp16, so that hi + lo * 2^-11 carries 22 bits of p; the
//     weights go from the scoring lanes (one key per lane, all heads) to the operand layout (one column per
//     lane, four keys) through 2 KB of LDS per wavefront, rows XOR-swizzled so that neither side conflicts;
//   * the accumulators (8 instructions x 4 registers) are rescaled only in tiles where a running maximum
//     moved; hi and lo columns are combined once, after the last tile.
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
constexpr float kLoScale = 2048.f;   // 2^11: lifts the remainder of a weight into fp16's normal range

template <int DK, int M, int CH, bool FUSED = false, int G = 1, bool MM = false>
__device__ __forceinline__ void consume_tile(const DecodeArgs &a, SoftmaxState<G> &st, const KeyCodes<M ? M : 4> &kc_in,
                                             v4u (&v)[CH], const float *lut_s, __amdgpu_buffer_rsrc_t rc,
                                             __amdgpu_buffer_rsrc_t rv, int bh, uint32_t kb, uint32_t k1,
                                             uint32_t kofs, int lane, int m, const double *enc_d,
                                             v4f (&accm)[MM ? 8 : 1], uint32_t pstage)
{
    constexpr int LPR = DK / 8;
    constexpr int NLD = LPR;
    const uint32_t key = kb + kofs;
    KeyCodes<M ? M : 4> kc = kc_in;
    if constexpr (FUSED) {
        // The newest key (row L-1) was encoded by this workgroup a moment ago: the lane that
        // scores it merges the per-wave minima, uses those codes and appends them to the cache.
        if (key == (uint32_t)(a.L - 1)) {
#pragma unroll
            for (int w = 0; w < (M + 3) / 4; ++w)
                kc.w[w] = 0u;
            const int *enc_c = reinterpret_cast<const int *>(enc_d + M * kDecWaves);
#pragma unroll
            for (int i = 0; i < M; ++i) {
                // waves hold ascending centroid ranges: strict '<' keeps the lowest index on ties
                double bd = enc_d[i * kDecWaves];
                int bc = enc_c[i * kDecWaves];
#pragma unroll
                for (int w = 1; w < kDecWaves; ++w) {
                    const double d = enc_d[i * kDecWaves + w];
                    const int c = enc_c[i * kDecWaves + w];
                    const bool better = d < bd;
                    bd = better ? d : bd;
                    bc = better ? c : bc;
                }
                kc.w[i / 4] |= (uint32_t)bc << (8 * (i % 4));
            }
            uint8_t *dst = a.codes_w + (int64_t)bh * a.code_stride + (int64_t)key * M;
            if constexpr (M == 2) {
                *reinterpret_cast<uint16_t *>(dst) = (uint16_t)kc.w[0];
            } else {
#pragma unroll
                for (int w = 0; w < M / 4; ++w)
                    reinterpret_cast<uint32_t *>(dst)[w] = kc.w[w];
            }
        }
    }
    // one score per query head of the group: the same codes index that head's tables
    float p[G];
    float corr_n = 1.f;      // MM: the correction of the query head whose column this lane accumulates
    bool moved = false;      // MM: some head's running maximum changed in this tile (wave-uniform)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float raw;
        if constexpr (M != 0)
            raw = kc.score(lut_s + g * (M * kCentroids));
        else
            raw = score_bytes(lut_s + g * (m * kCentroids), rc, key * m, m);
        float s = -INFINITY;
        if (key < k1) {
            if (a.scores_out)
                a.scores_out[((int64_t)bh * G + g) * a.L + key] = raw;
            s = raw * a.scale_log2e;
        }
        const float m_new = fmaxf(st.m_run[g], wave_max(s));
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = fast_exp2(st.m_run[g] - m_use);
        p[g] = fast_exp2(s - m_use);
        st.z[g] = st.z[g] * corr + p[g];
        if constexpr (MM) {
            corr_n = ((lane & (G - 1)) == g) ? corr : corr_n;
            moved = moved || (m_new != st.m_run[g]);
        } else {
#pragma unroll
            for (int d = 0; d < 8; ++d)
                st.acc[g][d] *= corr;
        }
        st.m_run[g] = m_new;
    }
    if constexpr (MM) {
        static_assert(DK == 128 && CH % 4 == 0 && G >= 4 && G <= 8, "matrix-core value sum: d_k = 128, 4 or 8 query heads");
        if (__builtin_amdgcn_readfirstlane((int)moved)) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                accm[e] *= corr_n;
        }
        // weights to the staging rows: this lane scored key 16*(sub/4) + 4*(sub%4) + rowin of the tile
        const uint32_t sub_ = (uint32_t)lane & 15u, rowin_ = (uint32_t)lane >> 4;
        const uint32_t r_w = (sub_ & ~3u) + rowin_;                 // staging row (step, rowin)
        const uint32_t w_base = pstage + r_w * 128u + 2u * (sub_ & 3u);
        const uint32_t w_swz = (r_w >> 1) * 8u;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const _Float16 hi = (_Float16)p[g];
            const _Float16 lo = (_Float16)((p[g] - (float)hi) * kLoScale);
            *reinterpret_cast<__attribute__((address_space(3))) _Float16 *>(w_base + (((uint32_t)g * 8u) ^ w_swz)) = hi;
            *reinterpret_cast<__attribute__((address_space(3))) _Float16 *>(w_base + (((uint32_t)(G + g) * 8u) ^ w_swz)) = lo;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t n_ = sub_, kg_ = rowin_;                    // operand column, contraction group
#pragma unroll
        for (int c0 = 0; c0 < NLD; c0 += CH) {
#pragma unroll
            for (int tt = 0; tt < CH / 4; ++tt) {
                const uint32_t r_r = (uint32_t)(c0 / 4 + tt) * 4u + kg_;
                const v4h bw = *reinterpret_cast<const __attribute__((address_space(3))) v4h *>(
                    pstage + r_r * 128u + ((n_ * 8u) ^ ((r_r >> 1) * 8u)));
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                    v2u aw;
                    aw.x = __builtin_amdgcn_perm(v[4 * tt + 1][e >> 1], v[4 * tt + 0][e >> 1], sel);
                    aw.y = __builtin_amdgcn_perm(v[4 * tt + 3][e >> 1], v[4 * tt + 2][e >> 1], sel);
                    accm[e] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(v4h, aw), bw, accm[e], 0, 0, 0);
                }
            }
            if (c0 + CH < NLD)
                load_rows<DK, CH>(v, rv, kb, c0 + CH, lane);   // next row groups of this tile
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();   // the next tile's weights overwrite the staging rows
        return;
    }
#pragma unroll
    for (int c0 = 0; c0 < NLD; c0 += CH) {
#pragma unroll
        for (int g = 0; g < G; ++g)   // the value rows are read once and weighted G times
            fma_rows<LPR, CH>(st.acc[g], p[g], v, c0);
        if (c0 + CH < NLD)
            load_rows<DK, CH>(v, rv, kb, c0 + CH, lane);   // next row groups of this tile
    }
}

// DK in {32, 64, 128, 256}; M in {2, 4, 8, 16} or 0 (= runtime m, byte loads);
// WAVES wavefronts per workgroup, OCC = wavefronts per SIMD the register budget must allow.
// Codebook rows of centroid `tid` for the GS subspaces i0 .. i0+GS-1 of one head.
template <int DSUB, int GS>
__device__ __forceinline__ void load_centroid_rows(float (&row)[GS][DSUB], const float *__restrict__ cb_head_c, int i0)
{
#pragma unroll
    for (int g = 0; g < GS; ++g) {
        const float *src = cb_head_c + (int64_t)(i0 + g) * kCentroids * DSUB;
        if constexpr (DSUB % 4 == 0) {
#pragma unroll
            for (int j4 = 0; j4 < DSUB / 4; ++j4) {
                const float4 t4 = reinterpret_cast<const float4 *>(src)[j4];
                row[g][4 * j4] = t4.x;
                row[g][4 * j4 + 1] = t4.y;
                row[g][4 * j4 + 2] = t4.z;
                row[g][4 * j4 + 3] = t4.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < DSUB; ++j)
                row[g][j] = src[j];
        }
    }
}

// Fused step, table-building wavefronts (256 threads): thread c takes centroid c of each subspace
// from the codebook of the head and from the same row computes
//   the table entry  LUT_i[c] = q^(i) . C_i[c]           (Sec. 3.5, fp32, ascending j)
//   the distance     || k_new^(i) - C_i[c] ||^2          (Sec. 3.4, fp64, as the encoder)
// and leaves per (subspace, wavefront) the smallest distance and its lowest centroid index in LDS.
// q and k_new are read-only and addressed uniformly over the wavefront: read through the constant
// address space they become scalar loads (SGPR operands of the FMAs below) and stay out of the
// in-order vector-memory queue.  Subspaces are processed in groups whose rows fit 64 registers,
// all rows of a group requested together.
// `encode`: this workgroup's range holds position L-1 (with several ranges per (b,h) only the last one
// scores the new key and appends its codes; the others build the table alone).
// G > 1 (grouped queries): bh is the key/value head; the G query heads bh*G .. bh*G+G-1 each get their
// table (lut_s[g][i][c]) from the one pass over the key/value head's codebook rows.
template <typename FT, int DK, int M, int G = 1, int NB = 1>
__device__ __forceinline__ void step_prologue(const DecodeArgs &a, int bh, int part, int tid, int lane, int wave,
                                              float *lut_s, double *enc_d, int *enc_c, int lds_stride, bool encode)
{
    // NB = 2 (two batch entries of one head per workgroup, each with its own 256 table builders): the builders
    // of entry `part` fetch the codebook rows of subspaces part*M/2 .. part*M/2 + M/2 - 1 only and from each row
    // compute the table entries and distances of BOTH entries (bh and bh + H; their LDS blocks lie lds_stride
    // bytes apart), so that the pair reads the head's codebook once instead of twice.
    static_assert(NB == 1 || (NB == 2 && G == 1 && M % 2 == 0), "paired batch entries: ungrouped, even m");
    constexpr int DSUB = DK / M;
    constexpr int MS = M / NB;            // subspaces this builder group covers
    // rows held at once: 64 registers; paired entries keep two entries' distances alive, so there short rows
    // (d_sub < 16) are taken 16 registers at a time and, at d_k = 128 (twice the tile registers), longer ones 32
    constexpr int kRowRegs = (NB == 2) ? ((DSUB < 16) ? 16 : (DK == 128 ? 32 : 64)) : 64;
    constexpr int GS0 = (kRowRegs / DSUB) < 1 ? 1 : ((kRowRegs / DSUB) > MS ? MS : (kRowRegs / DSUB));
    constexpr int GS = (MS % GS0 == 0) ? GS0 : 1;
    float frow[GS][DSUB];
    const int ibase = part * MS;
    const float *__restrict__ cbh = a.codebooks + (int64_t)(bh % a.H) * M * kCentroids * DSUB + (int64_t)tid * DSUB;
    UniformWords qg[NB], kg[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const uintptr_t row = (uintptr_t)(bh + nb * a.H);
        qg[nb] = (UniformWords)(reinterpret_cast<uintptr_t>(a.q) + row * G * DK * sizeof(FT));
        kg[nb] = (UniformWords)(reinterpret_cast<uintptr_t>(a.k_new) + row * DK * sizeof(FT));
    }
    // The scalar loads of q and k_new are issued a subspace at a time, each shortly before its use, and
    // the rows are cold (written by the previous layer's kernels): every 128-byte line would cost a
    // memory round trip in the middle of the table arithmetic.  One word of every line is requested
    // here, ahead of the codebook rows, so that those loads find the lines in L2.
    // (Ungrouped only: with grouped queries, whose workgroups stream megabytes each, it measured slower.)
    uint32_t touched = 0;
    if constexpr (G == 1) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int o = 0; o < (int)(DK * sizeof(FT)); o += 128)
                touched |= qg[nb][o / 4];
#pragma unroll
            for (int o = 0; o < (int)(DK * sizeof(FT)); o += 128)
                touched |= kg[nb][o / 4];
        }
    }
    load_centroid_rows<DSUB, GS>(frow, cbh, ibase);
#pragma unroll
    for (int i0 = 0; i0 < MS; i0 += GS) {
        if (i0 > 0)
            load_centroid_rows<DSUB, GS>(frow, cbh, ibase + i0);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float *lut_nb = reinterpret_cast<float *>(reinterpret_cast<char *>(lut_s) + nb * lds_stride);
            double *encd_nb = reinterpret_cast<double *>(reinterpret_cast<char *>(enc_d) + nb * lds_stride);
            int *encc_nb = reinterpret_cast<int *>(reinterpret_cast<char *>(enc_c) + nb * lds_stride);
            double dv[GS], dm[GS];
#pragma unroll
            for (int g = 0; g < GS; ++g) {
                const int i = ibase + i0 + g;
#pragma unroll
                for (int hq = 0; hq < G; ++hq) {
                    float e = 0.f;
#pragma unroll
                    for (int j = 0; j < DSUB; ++j)
                        e = fmaf(uniform_elem<FT>(qg[nb], hq * DK + i * DSUB + j), frow[g][j], e);
                    lut_nb[(hq * M + i) * kCentroids + tid] = e;
                }
                if (G == 1 || encode) {
                    dv[g] = argmin_value(step_sq_dist<FT, DSUB>(kg[nb], i * DSUB, frow[g]), tid);
                    dm[g] = dv[g];
                }
            }
            // Ungrouped, the distances are evaluated in every range and published only where the new key is
            // scored: the branch would cost more than the arithmetic.  With grouped queries the ranges that
            // do not hold the new key skip them (eight heads' tables already keep those wavefronts busy).
            if (G == 1 || encode) {
                dmin_wave<GS>(dm);
#pragma unroll
                for (int g = 0; g < GS; ++g) {
                    // lowest lane that holds the wave minimum = lowest centroid index of this wave
                    const uint64_t holders = __ballot(dv[g] == dm[g]);
                    if (lane == 0 && encode) {
                        encd_nb[(ibase + i0 + g) * kDecWaves + wave] = dm[g];
                        encc_nb[(ibase + i0 + g) * kDecWaves + wave] = wave * kWave + (int)__builtin_ctzll(holders);
                    }
                }
            }
        }
    }
    asm volatile("" ::"s"(touched));   // keeps the early requests alive; nothing reads them
}

// FT = void: the table comes from memory (lookat_attend_decode).  FT = __half / float: fused
// decode step (lookat_decode_step): q and the new key have type FT, the table is computed and
// the new key encoded by the workgroup itself (WAVES = 8; see the roles below).
// G > 1: grouped-query attention: the workgroup's (b,h) is a KEY/VALUE head shared by G query heads,
// whose tables (contiguous in memory) are all staged in LDS; codes and values are streamed once.
// PF: tiles of a wavefront requested before anything else is done (1, or more for the fused step,
// whose table build and key encoding would otherwise leave the memory pipe idle for microseconds).
// NB = 2 (fused step only): the workgroup has 2 x WAVES wavefronts and serves TWO batch entries of one head,
// (b, h) and (b + 1, h).  Each half is a complete copy of the roles above with its own LDS block; the only
// thing shared is the codebook, of which each half's table builders fetch half the subspaces and compute
// both entries' table rows and distances.  The head's codebook then crosses from L2 to the compute units
// once per pair instead of once per (b,h).  Both halves execute the same barriers (same L, same ranges).
template <int DK, int M, int WAVES, int OCC, typename FT = void, int G = 1, int PF = 1, int NB = 1>
__global__ __launch_bounds__(WAVES *NB *kWave, OCC) void decode_split_kernel(LOOKAT_DECODE_HEAD_PARAMS,
                                                                             const DecodeLate late)
{
    const DecodeArgs a = rebuild_args(p_BH, p_splits, p_H, p_table, p_codes, p_values, p_code_stride, p_value_stride,
                                      p_L, p_kps, p_scale_log2e, late, !std::is_void<FT>::value);
    constexpr bool FUSED = !std::is_void<FT>::value;
    static_assert(!FUSED || (WAVES == 2 * kDecWaves && M != 0), "fused step: 512 threads, compile-time m");
    static_assert(NB == 1 || (NB == 2 && FUSED && G == 1), "paired batch entries: ungrouped fused step only");
    // Fused step: the eight wavefronts take two roles until the table exists.  The first four
    // (256 threads, thread c = centroid c) fetch the codebook rows, build the table and encode the
    // new key (step_prologue) and request no tile before that is done; the other four request
    // their tiles at once and wait.  A wavefront issues in order, and under a saturated memory
    // pipe a tile request is accepted only as fast as data leaves the pipe: a wavefront that has
    // tile requests queued ahead of its table arithmetic starts that arithmetic microseconds late.
    static_assert(G == 1 || M != 0, "grouped queries: compile-time m");
    constexpr int LPR = DK / 8;            // lanes per value row (16 bytes per lane)
    constexpr int RPL = kWave / LPR;       // value rows covered by one wave-wide load
    constexpr int NLD = kTile / RPL;       // wave-wide loads per tile (= LPR)
    constexpr bool MM = (G >= 4 && DK == 128 && M != 0);   // weighted value sum on the matrix cores
    // loads kept in flight together: 8 KB of a tile; the whole 16 KB tile where the matrix cores take the value sum
    // (its accumulators are half the size, and a second request round in the middle of a tile is a second
    // exposed round trip at two wavefronts per SIMD)
    constexpr int CH = MM ? NLD : (NLD < 8 ? NLD : 8);
    constexpr int NT = WAVES * kWave;

    extern __shared__ __align__(16) float smem_all[];
    // which of the workgroup's NB batch entries this wavefront belongs to (scalar), and its LDS block
    const int hf = (NB == 1) ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / (WAVES * kWave));
    constexpr int kHalfBytes = (NB == 1) ? 0 : (int)step_pair_lds_bytes(M, DK);
    float *smem = reinterpret_cast<float *>(reinterpret_cast<char *>(smem_all) + hf * kHalfBytes);
    float *lut_s = smem;                                   // [G][m][256]
    float *red_s = smem + G * (M ? M : a.m) * kCentroids;  // [WAVES][G][DK + 2]
    double *enc_d = reinterpret_cast<double *>(red_s + WAVES * G * (DK + 2));   // fused step: [M][WAVES] minima,
    int *enc_c = reinterpret_cast<int *>(enc_d + (M ? M : 1) * kDecWaves);     //             then [M][WAVES] indices

    int bh, split;
    if constexpr (NB == 1) {
        if (!map_block(a, bh, split))
            return;
    } else {
        // a.BH / 2 pairs are dealt to the workgroups as (b,h) pairs are otherwise: pair p = head p % H of the
        // batch entries 2*(p / H) and 2*(p / H) + 1
        int pair;
        if (!map_block_n(a, a.BH / 2, pair, split))
            return;
        bh = 2 * (pair / a.H) * a.H + pair % a.H + hf * a.H;
    }
    const int m = M ? M : a.m;
    const int tid = (NB == 1) ? (int)threadIdx.x : (int)threadIdx.x - hf * (WAVES * kWave);   // within the half
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // in a scalar register: role branches are scalar branches
    const bool builds_table = FUSED && wave < kDecWaves;

    const uint32_t k0 = (uint32_t)split * (uint32_t)a.keys_per_split;
    const uint32_t k1 = (k0 + a.keys_per_split < a.L) ? (uint32_t)(k0 + a.keys_per_split) : (uint32_t)a.L;
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(a.values + (int64_t)bh * a.value_stride, k1 * (uint32_t)(DK * 2));
    const __amdgpu_buffer_rsrc_t rc = make_rsrc(a.codes + (int64_t)bh * a.code_stride, k1 * (uint32_t)m);

    // Everything the first tile needs is requested before anything is waited for, in the
    // order it is needed (loads return in order, so each wait below covers only what precedes):
    // 1) this thread's slice of the table (staged through registers: the wait before the
    //    barrier then covers the table alone, not the value rows behind it);
    const float4 *lut_g = reinterpret_cast<const float4 *>(a.lut + (int64_t)bh * G * m * kCentroids);
    constexpr int kLutRegs = M ? (G * M * (kCentroids / 4) + NT - 1) / NT : 1;
    // (tables of more than one 16-byte piece per thread are copied up front instead: a staging
    // array of several registers ends up in scratch memory)
    constexpr bool STAGED = (M != 0 && !FUSED && kLutRegs == 1);
    float4 lut_r[STAGED ? kLutRegs : 1];
    if constexpr (M != 0 && !FUSED && !STAGED) {
        float4 *s4 = reinterpret_cast<float4 *>(lut_s);
        for (int x = tid; x < G * M * (kCentroids / 4); x += NT)
            s4[x] = lut_g[x];
    }
    if constexpr (STAGED) {
#pragma unroll
        for (int x = 0; x < kLutRegs; ++x)
            if ((x + 1) * NT <= G * M * (kCentroids / 4) || tid + x * NT < G * M * (kCentroids / 4))
                lut_r[x] = lut_g[tid + x * NT];
            else
                lut_r[x] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    // 2) the codes of the wave's first tile;  3) its value rows.
    // Lane (rowin, sub) holds the value rows RPL*j + rowin, j = 0..NLD-1, of a tile.  It scores
    // the key RPL*sub + rowin, so the NLD weights a lane needs sit in its own group of LPR
    // consecutive lanes and are fetched with DPP moves instead of LDS shuffles.
    const int sub = lane % LPR;      // which 8-coordinate slice of the value row
    const int rowin = lane / LPR;    // which row of a wave-wide load
    const uint32_t kofs = (uint32_t)(RPL * sub + rowin);
    uint32_t kb = k0 + (uint32_t)wave * kTile;
    KeyCodes<M ? M : 4> kcs[PF];
    v4u vs[PF][CH];
    // Unconditional within its role: requests past the range return zero (descriptor bounds).  Behind a
    // per-tile branch the compiler could no longer count how many requests follow a given one, and every
    // wait would become a wait for all of them.  (A macro: a lambda that captures the register arrays
    // sends them through scratch memory.)
#define LOOKAT_REQUEST_FIRST_TILES()                                                                   \
    _Pragma("unroll") for (int t = 0; t < PF; ++t)                                                     \
    {                                                                                                  \
        const uint32_t kbt = kb + (uint32_t)t * NT;                                                    \
        if constexpr (M != 0)                                                                          \
            kcs[t].load(rc, (kbt + kofs) * M);                                                         \
        __builtin_amdgcn_sched_barrier(0); /* keep the request order: codes before value rows */       \
        load_rows<DK, CH>(vs[t], rv, kbt, 0, lane);                                                    \
    }
    if constexpr (FUSED) {
        // one branch per role: the table builders' codebook rows and the streamers' tiles then never
        // hold registers at the same time
        if (builds_table) {
            // issue ahead of the streamers that share the SIMD: the codebook requests must enter the
            // compute unit's memory queue before the tile requests fill it
            __builtin_amdgcn_s_setprio(3);
            // (paired entries: the LDS blocks and the (b,h) index are handed over as entry 0's)
            step_prologue<FT, DK, M, G, NB>(a, bh - hf * a.H, hf, tid, lane, wave,
                                            reinterpret_cast<float *>(reinterpret_cast<char *>(lut_s) - hf * kHalfBytes),
                                            reinterpret_cast<double *>(reinterpret_cast<char *>(enc_d) - hf * kHalfBytes),
                                            reinterpret_cast<int *>(reinterpret_cast<char *>(enc_c) - hf * kHalfBytes),
                                            kHalfBytes, k1 == (uint32_t)a.L);
            __builtin_amdgcn_s_setprio(0);
        } else {
            LOOKAT_REQUEST_FIRST_TILES()
        }
    } else {
        LOOKAT_REQUEST_FIRST_TILES()
    }
    KeyCodes<M ? M : 4> &kc = kcs[0];
    v4u(&v)[CH] = vs[0];
    if constexpr (!FUSED) {
        float4 *s4 = reinterpret_cast<float4 *>(lut_s);
        if constexpr (STAGED) {
#pragma unroll
            for (int x = 0; x < kLutRegs; ++x)
                if ((x + 1) * NT <= G * M * (kCentroids / 4) || tid + x * NT < G * M * (kCentroids / 4))
                    s4[tid + x * NT] = lut_r[x];
        } else if constexpr (M == 0) {
            for (int x = tid; x < m * (kCentroids / 4); x += NT)
                s4[x] = lut_g[x];
        }
    }
    __syncthreads();   // table (and, fused, the per-wave argmins) complete in LDS; value rows stay in flight
    if constexpr (FUSED) {
        if (builds_table) {
            LOOKAT_REQUEST_FIRST_TILES()
        }
    }
#undef LOOKAT_REQUEST_FIRST_TILES

    // First tile (requested above), then the wave's remaining tiles: request, consume.  Tiles
    // are requested only if they exist (a load past the range would return zero but still
    // occupy the address pipeline), and a tile's registers are dead at the loop back-edge.
    SoftmaxState<G> st;
    // Matrix-core value sum (see consume_tile): accumulators, and the wavefront's weight staging rows, which
    // occupy its own slice of the reduction buffer (unused until the epilogue; 2 KB of its G x (DK + 2) floats).
    v4f accm[MM ? 8 : 1];
#pragma unroll
    for (int e = 0; e < (MM ? 8 : 1); ++e)
        accm[e] = v4f{0.f, 0.f, 0.f, 0.f};
    uint32_t pstage = 0;
    if constexpr (MM) {
        static_assert(G * (DK + 2) * sizeof(float) >= 2048, "the staging rows fit the wavefront's reduction slice");
        pstage = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float *)(red_s + wave * G * (DK + 2));
        // columns no query head owns (G = 4: 8..15) must read as zero in every tile
        *reinterpret_cast<__attribute__((address_space(3))) v4f *>(pstage + (uint32_t)lane * 32u) = v4f{0.f, 0.f, 0.f, 0.f};
        *reinterpret_cast<__attribute__((address_space(3))) v4f *>(pstage + (uint32_t)lane * 32u + 16u) = v4f{0.f, 0.f, 0.f, 0.f};
    }
    if (kb < k1) {
        consume_tile<DK, M, CH, FUSED, G, MM>(a, st, kc, v, lut_s, rc, rv, bh, kb, k1, kofs, lane, m, enc_d, accm, pstage);
#pragma unroll
        for (int t = 1; t < PF; ++t) {   // the other tiles requested at the start
            kb += NT;
            if (kb < k1)
                consume_tile<DK, M, CH, FUSED, G, MM>(a, st, kcs[t], vs[t], lut_s, rc, rv, bh, kb, k1, kofs, lane, m, enc_d, accm,
                                                      pstage);
        }
        for (kb += NT; kb < k1; kb += NT) {
            if constexpr (M != 0)
                kc.load(rc, (kb + kofs) * M);
            __builtin_amdgcn_sched_barrier(0);   // request order = need order: codes before value rows
            load_rows<DK, CH>(v, rv, kb, 0, lane);
            consume_tile<DK, M, CH, FUSED, G, MM>(a, st, kc, v, lut_s, rc, rv, bh, kb, k1, kofs, lane, m, enc_d, accm, pstage);
        }
    }

    // ---- fold the rows of the wave, then the waves of the workgroup ----
    if constexpr (MM) {
        // lane (q, n): accm[e][r] = coordinate 8*(4q + r) + e of column n; columns n < G hold the fp16 part of
        // the weights, columns G + n the scaled remainder: combine, and lanes n < G hand over head n's sum
        const int n = lane & 15, q = lane >> 4;
        float *mine_n = red_s + (wave * G + (n & (G - 1))) * (DK + 2);
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float lo = dpp_mov<0x100 + G>(accm[e][r], accm[e][r]);   // row_shl:G -- lane n + G of the row
                const float o = fmaf(lo, 1.f / kLoScale, accm[e][r]);
                if (n < G)
                    mine_n[8 * (4 * q + r) + e] = o;
            }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if constexpr (!MM) {
#pragma unroll
            for (int d = 0; d < 8; ++d)
                st.acc[g][d] = sum_over_lane_classes<LPR>(st.acc[g][d]);
        }
        st.z[g] = wave_sum(st.z[g]);
        float *mine = red_s + (wave * G + g) * (DK + 2);
        if constexpr (!MM) {
            if (lane < LPR) {
#pragma unroll
                for (int d = 0; d < 8; ++d)
                    mine[sub * 8 + d] = st.acc[g][d];
            }
        }
        if (lane == 0) {
            mine[DK] = st.m_run[g];
            mine[DK + 1] = st.z[g];
        }
    }
    __syncthreads();

    auto finish = [&](int x) {   // x = (query head of the group, output coordinate)
        const int g = x / DK, j = x % DK;
        float mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < WAVES; ++w)
            mx = fmaxf(mx, red_s[(w * G + g) * (DK + 2) + DK]);
        const float m_use = (mx == -INFINITY) ? 0.f : mx;
        float o = 0.f, zz = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float wgt = fast_exp2(red_s[(w * G + g) * (DK + 2) + DK] - m_use);
            o = fmaf(wgt, red_s[(w * G + g) * (DK + 2) + j], o);
            zz = fmaf(wgt, red_s[(w * G + g) * (DK + 2) + DK + 1], zz);
        }
        if (a.splits == 1) {
            a.out[((int64_t)bh * G + g) * DK + j] = o / zz;
        } else {
            float *dst = a.part + (((int64_t)bh * G + g) * a.splits + split) * (DK + 2);
            dst[j] = o;
            if (j == 0) {
                dst[DK] = mx;
                dst[DK + 1] = zz;
            }
        }
    };
    if constexpr (G * DK <= NT) {
        if (tid < G * DK)
            finish(tid);
    } else {
        for (int x = tid; x < G * DK; x += NT)
            finish(x);
    }
}

// Any d_k (multiple of 8, <= 256) and any m: one 256-key tile per step, scores through LDS,
// thread j owns output coordinate j.  Used for head dimensions without a tuned kernel.
__global__ __launch_bounds__(kDecThreads) void decode_split_generic_kernel(LOOKAT_DECODE_HEAD_PARAMS,
                                                                           const DecodeLate late)
{
    const DecodeArgs a = rebuild_args(p_BH, p_splits, p_H, p_table, p_codes, p_values, p_code_stride, p_value_stride,
                                      p_L, p_kps, p_scale_log2e, late, false);
    extern __shared__ __align__(16) float smem[];
    float *lut_s = smem;                          // [m][256]
    float *p_s = smem + a.m * kCentroids;         // [256] scores -> weights of the tile
    float *red_s = p_s + kDecThreads;             // [kDecWaves]

    int bh, split;
    if (!map_block(a, bh, split))
        return;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int m = a.m, d_k = a.d_k;

    for (int x = tid; x < m * kCentroids; x += kDecThreads)
        lut_s[x] = a.lut[(int64_t)bh * m * kCentroids + x];
    __syncthreads();

    const int64_t k0 = (int64_t)split * a.keys_per_split;
    const int64_t k1 = (k0 + a.keys_per_split < a.L) ? (k0 + a.keys_per_split) : a.L;
    const uint8_t *codes_bh = a.codes + (int64_t)bh * a.code_stride;
    const __half *values_bh = a.values + (int64_t)bh * a.value_stride;

    float m_run = -INFINITY, z = 0.f, o = 0.f;
    for (int64_t kb = k0; kb < k1; kb += kDecThreads) {
        const int64_t key = kb + tid;
        float s = -INFINITY;
        if (key < k1) {
            float raw = 0.f;
            for (int i = 0; i < m; ++i)
                raw += lut_s[i * kCentroids + codes_bh[key * m + i]];
            if (a.scores_out)
                a.scores_out[(int64_t)bh * a.L + key] = raw;
            s = raw * a.scale_log2e;
        }
        const float wm = wave_max(s);
        if (lane == 0)
            red_s[wave] = wm;
        __syncthreads();
        float tmax = red_s[0];
#pragma unroll
        for (int w = 1; w < kDecWaves; ++w)
            tmax = fmaxf(tmax, red_s[w]);
        const float m_new = fmaxf(m_run, tmax);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = fast_exp2(m_run - m_use);
        p_s[tid] = fast_exp2(s - m_use);
        __syncthreads();
        const int cnt = (int)((k1 - kb < kDecThreads) ? (k1 - kb) : kDecThreads);
        float zt = 0.f;
        for (int r = 0; r < cnt; ++r)
            zt += p_s[r];
        z = z * corr + zt;
        o *= corr;
        if (tid < d_k) {
            for (int r = 0; r < cnt; ++r)
                o = fmaf(p_s[r], __half2float(values_bh[(kb + r) * d_k + tid]), o);
        }
        m_run = m_new;
        __syncthreads();
    }
    if (tid < d_k) {
        if (a.splits == 1) {
            a.out[(int64_t)bh * d_k + tid] = o / z;
        } else {
            float *dst = a.part + ((int64_t)bh * a.splits + split) * (d_k + 2);
            dst[tid] = o;
            if (tid == 0) {
                dst[d_k] = m_run;
                dst[d_k + 1] = z;
            }
        }
    }
}

// Merge of the split ranges: M* = max_s M_s, out = sum_s 2^(M_s-M*) o_s / sum_s 2^(M_s-M*) Z_s.
// An empty range carries (M=-inf, Z=0, o=0) and gets weight 0.
// The ranges are taken eight at a time with all of a group's loads issued before the first is used: a loop
// that loads and uses one range per iteration pays one memory round trip per range (8 ranges: 5.2 us for a
// kernel that moves 130 floats per range).  Up to eight ranges the sums are formed exactly as a plain
// ascending loop would; beyond, the running sums are rescaled when a later group raises the maximum.
//   grid = BH, block = 256 (threads >= d_k idle)
__global__ __launch_bounds__(kDecThreads) void decode_combine_kernel(const float *__restrict__ part,
                                                                     float *__restrict__ out, int splits, int d_k)
{
    constexpr int GR = 8;
    const int bh = blockIdx.x;
    const int tid = threadIdx.x;
    if (tid >= d_k)
        return;
    const float *p = part + (int64_t)bh * splits * (d_k + 2);
    float mx = -INFINITY, o = 0.f, z = 0.f;
    for (int s0 = 0; s0 < splits; s0 += GR) {
        float mv[GR], zv[GR], ov[GR];
#pragma unroll
        for (int j = 0; j < GR; ++j) {
            const bool live = s0 + j < splits;
            const float *ps = p + (int64_t)(live ? s0 + j : s0) * (d_k + 2);
            const float m_ = ps[d_k], z_ = ps[d_k + 1], o_ = ps[tid];
            mv[j] = live ? m_ : -INFINITY;
            zv[j] = live ? z_ : 0.f;
            ov[j] = live ? o_ : 0.f;
        }
        float gm = mx;
#pragma unroll
        for (int j = 0; j < GR; ++j)
            gm = fmaxf(gm, mv[j]);
        const float m_use = (gm == -INFINITY) ? 0.f : gm;
        const float keep = fast_exp2(mx - m_use);     // 0 for the first group (mx = -inf), 1 when the maximum stays
        o *= keep;
        z *= keep;
#pragma unroll
        for (int j = 0; j < GR; ++j) {
            const float w = fast_exp2(mv[j] - m_use);
            o = fmaf(w, ov[j], o);
            z = fmaf(w, zv[j], z);
        }
        mx = gm;
    }
    out[(int64_t)bh * d_k + tid] = o / z;
}

static int64_t round_up(int64_t x, int64_t q) { return (x + q - 1) / q * q; }

// Ranges per (b,h) when the caller leaves the choice to the library.  One range as long as the
// (b,h) count alone fills the 256 compute units: the merge kernel is a second launch and costs more
// than it buys on short contexts.  With fewer (b,h) pairs the sequence is cut so that about
// `workgroups` workgroups exist, but never into ranges shorter than `min_range` keys.
static int auto_splits(const lookat_shape *s, int64_t L, int workgroups = 256, int min_range = 2048)
{
    // Ungrouped kernels: one workgroup per compute unit and ranges of at least 2048 keys, measured
    // at d_k = 128, m = 8 (us per call, 2/4/8/16 ranges): 32 (b,h) x 32768 keys: -/55/54/60;
    // 64 x 32768: 103/95/99/107; 128 x 32768: 183/183/190/-; 32 x 8192: 25.8/18.7/20.4/24.6.
    const int64_t BH = (int64_t)s->B * s->H;
    int64_t want = workgroups / BH;
    const int64_t cap = (L + min_range - 1) / min_range;
    if (want > cap)
        want = cap;
    if (want < 1)
        want = 1;
    if (want > 256)
        want = 256;
    return (int)want;
}
// Grouped queries: from group 4 on one 512-thread workgroup per compute unit (see gqa_waves), at
// group 2 two 256-thread ones.  Measured at 8 x 32 query heads x 32768 keys, d_k = 128, m = 8 (us per
// launch at 128 / 256 / 512 / 1024 workgroups): group 4: 148 / 102 / 111 / 113; group 8: 127 / 75 / 84 / 102;
// group 2: 283 / 187 / 186 / 200.
static int auto_splits_gqa(const lookat_shape *s, int group, int64_t L)
{
    return group >= 4 ? auto_splits(s, L, 256, 1024) : auto_splits(s, L, 512, 1024);
}

static bool tuned_dk(int d_k) { return d_k == 32 || d_k == 64 || d_k == 128 || d_k == 256; }

template <int DK, int WAVES, int OCC>
static void launch_tuned(const DecodeArgs &a, dim3 grid, hipStream_t st)
{
    dim3 block(WAVES * kWave);
    const size_t lds = ((size_t)a.m * kCentroids + (size_t)WAVES * (DK + 2)) * sizeof(float);
    switch (a.m) {
    case 2:
        hipLaunchKernelGGL((decode_split_kernel<DK, 2, WAVES, OCC>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, false),
                           late_of(a));
        break;
    case 4:
        hipLaunchKernelGGL((decode_split_kernel<DK, 4, WAVES, OCC>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, false),
                           late_of(a));
        break;
    case 8:
        hipLaunchKernelGGL((decode_split_kernel<DK, 8, WAVES, OCC>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, false),
                           late_of(a));
        break;
    case 16:
        hipLaunchKernelGGL((decode_split_kernel<DK, 16, WAVES, OCC>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, false),
                           late_of(a));
        break;
    default:
        hipLaunchKernelGGL((decode_split_kernel<DK, 0, WAVES, OCC>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, false),
                           late_of(a));
        break;
    }
}

// Wavefronts per workgroup: 16 for long ranges (at least 32 tiles), else 4 (measured on
// MI355X: the small workgroup wins at context 1024, the large one from 16K keys on).
static int pick_waves(int d_k, int m, int64_t keys_per_split)
{
    if ((d_k != 64 && d_k != 128) || (m != 2 && m != 4 && m != 8))
        return 4;   // the 16-wave variant must fit 64 registers; only these shapes do
    return keys_per_split >= 32 * kTile ? 16 : 4;
}

// Fused decode step: one workgroup of 512 threads per (b,h), one range: four wavefronts build the
// table and encode the new key, four request their first kStepPrefetch tiles at once; after the
// barrier the table builders request theirs and all eight stream.  Measured at B=32, H=12,
// L=1024, m=4 (us per launch): 256 threads, every wavefront doing both 13.8 (one tile ahead 14.0,
// four 15.9); 512 threads with the two roles 13.4; the same with the table builders at raised
// wave priority 11.8 (their codebook requests enter the compute unit's memory queue ahead of
// the streamers' tile requests instead of interleaved with them).
constexpr int kStepPrefetch = 2;
constexpr int kStepWaves = 2 * kDecWaves;   // four wavefronts build the table, four start streaming at once
template <int DK, typename FT>
static bool launch_step(const DecodeArgs &a, dim3 grid, hipStream_t st)
{
    dim3 block(kStepWaves * kWave);
    const size_t lds = ((size_t)a.m * kCentroids + (size_t)kStepWaves * (DK + 2)) * sizeof(float) +
                       (size_t)a.m * kDecWaves * (sizeof(double) + sizeof(int));
    switch (a.m) {
    case 2:
        hipLaunchKernelGGL((decode_split_kernel<DK, 2, kStepWaves, 4, FT, 1, kStepPrefetch>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, true),
                           late_of(a));
        return true;
    case 4:
        hipLaunchKernelGGL((decode_split_kernel<DK, 4, kStepWaves, 4, FT, 1, kStepPrefetch>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, true),
                           late_of(a));
        return true;
    case 8:
        hipLaunchKernelGGL((decode_split_kernel<DK, 8, kStepWaves, 4, FT, 1, kStepPrefetch>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, true),
                           late_of(a));
        return true;
    case 16:
        hipLaunchKernelGGL((decode_split_kernel<DK, 16, kStepWaves, 4, FT, 1, 1>), grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, true),
                           late_of(a));
        return true;
    default:
        return false;
    }
}

// Two batch entries of one head per workgroup (1024 threads): see decode_split_kernel, NB = 2.
// When the library takes it.  A compute unit holds two 512-thread workgroups of the fused step or one paired
// one, and a launch is as slow as its most loaded compute unit.  Up to 256 (b,h) every workgroup has a
// compute unit to itself and pairing only halves the parallelism (192 (b,h) x 1024 keys, d_k = 64, m = 4,
// graph replays: 7.2 us single, 9.5 us paired); from 257 to 512 (b,h) some compute units carry two (b,h)
// either way and the pairs halve the codebook traffic (264: 11.0 -> 9.8 us; 384: 11.8 -> 11.0; 504:
// 14.4 -> 13.0); beyond 512 the pairs need a second round of workgroups where single entries still
// fit two to a compute unit (528: 17.7 single, 20.3 paired).  Short contexts (512 keys: 8.8 / 8.9 us) and m >= 8
// (m = 8: 11.4 / 11.8 us; m = 16: 14.4 / 15.1) measured no gain at d_k = 64.
// d_k = 128 (fp16 queries, graph replays, single / paired us): m = 4: 384 (b,h) x 1024 keys 23.7 / 22.3, 512 x 1024
// 30.8 / 27.1, 320 x 1024 23.3 / 20.4, 384 x 4096 72.6 / 66.7, 512 x 512 20.2 / 17.9; m = 8: 384 x 1024 21.6 / 22.3,
// 512 x 1024 27.4 / 26.6, 512 x 512 17.3 / 17.5, 384 x 4096 71.9 / 69.5, 320 x 2048 38.3 / 33.4, 512 x 2048 (fp32)
// 51.2 / 49.3: taken from 2048 keys on; m = 16: 384 x 1024 23.7 / 24.8, 512 x 1024 27.8 / 30.2: not taken;
// m = 2 (one codebook row = 64 registers) has no paired instance at d_k = 128: it would spill.
static bool step_pairs_entries(const lookat_shape *s, int group, int64_t L, int S)
{
    const int64_t BH = (int64_t)s->B * s->H;
    if (group != 1 || S != 1 || (s->B & 1) || BH <= 256 || BH > 512)
        return false;
    if (s->d_k == 64)
        return (s->m == 2 || s->m == 4) && L >= 768;
    if (s->d_k == 128)
        return (s->m == 4 && L >= 512) || (s->m == 8 && L >= 2048);
    return false;
}

template <int DK, typename FT>
static bool launch_step_pair(const DecodeArgs &a, dim3 grid, hipStream_t st)
{
    dim3 block(2 * kStepWaves * kWave);
    const size_t lds = 2 * step_pair_lds_bytes(a.m, DK);
    switch (a.m) {
    case 2:
        if constexpr (DK == 64) {
            hipLaunchKernelGGL((decode_split_kernel<DK, 2, kStepWaves, 4, FT, 1, kStepPrefetch, 2>), grid, block, lds, st,
                               LOOKAT_DECODE_HEAD_ARGS(a, true), late_of(a));
            return true;
        }
        return false;
    case 4:
        hipLaunchKernelGGL((decode_split_kernel<DK, 4, kStepWaves, 4, FT, 1, kStepPrefetch, 2>), grid, block, lds, st,
                           LOOKAT_DECODE_HEAD_ARGS(a, true), late_of(a));
        return true;
    case 8:
        hipLaunchKernelGGL((decode_split_kernel<DK, 8, kStepWaves, 4, FT, 1, kStepPrefetch, 2>), grid, block, lds, st,
                           LOOKAT_DECODE_HEAD_ARGS(a, true), late_of(a));
        return true;
    case 16:
        hipLaunchKernelGGL((decode_split_kernel<DK, 16, kStepWaves, 4, FT, 1, 1, 2>), grid, block, lds, st,
                           LOOKAT_DECODE_HEAD_ARGS(a, true), late_of(a));
        return true;
    default:
        return false;
    }
}

// Grouped queries: 256-thread workgroups; four wavefronts per SIMD up to G = 4 (G accumulator sets
// per lane fit 128 registers), two for G = 8.
// LDS of a grouped-query workgroup: the group's tables and the per-wavefront partial results.
static size_t gqa_lds_bytes(int group, int m, int d_k, int waves)
{
    return ((size_t)group * m * kCentroids + (size_t)waves * group * (d_k + 2)) * sizeof(float);
}
// From group 4 on a workgroup has eight wavefronts where LDS allows: two wavefronts per SIMD share one
// copy of the group's tables (group x m KB) instead of two four-wavefront workgroups holding a copy
// each.  B=8, 32 query heads, 32768 keys, d_k=128, m=8: group 8: 81 us against 97 us; group 4: 102
// against 115 us.
static int gqa_waves(int group, int m, int d_k)
{
    return (group >= 4 && gqa_lds_bytes(group, m, d_k, 2 * kDecWaves) <= 160 * 1024) ? 2 * kDecWaves : kDecWaves;
}

template <int DK, int G, int GW = kDecWaves>
static int launch_gqa(const DecodeArgs &a, dim3 grid, hipStream_t st)
{
    dim3 block(GW * kWave);
    const size_t lds = gqa_lds_bytes(G, a.m, DK, GW);
#define LOOKAT_GQA_CASE(M_)                                                                                    \
    case M_: {                                                                                                 \
        auto kern = decode_split_kernel<DK, M_, GW, ((DK == 128 && G >= 4) ? 2 : (G <= 4 ? 4 : (GW == kDecWaves ? 3 : 2))), void, G>; \
        if (lds > 64 * 1024) {                                                                                 \
            /* allow more than 64 KB of dynamic LDS: idempotent, so every call makes it (no shared flag) */   \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                          \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);         \
            if (e != hipSuccess)                                                                               \
                return fail(LOOKAT_ERR_HIP, "lookat_attend_decode_gqa: cannot reserve %zu bytes of LDS: %s", lds, \
                            hipGetErrorString(e));                                                             \
        }                                                                                                      \
        hipLaunchKernelGGL(kern, grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, false), late_of(a));         \
        return LOOKAT_OK;                                                                                      \
    }
    switch (a.m) {
        LOOKAT_GQA_CASE(2)
        LOOKAT_GQA_CASE(4)
        LOOKAT_GQA_CASE(8)
        LOOKAT_GQA_CASE(16)
    default:
        return fail(LOOKAT_ERR_UNSUPPORTED, "lookat_attend_decode_gqa handles m in {2,4,8,16}; got m=%d", a.m);
    }
#undef LOOKAT_GQA_CASE
}

// Fused step with grouped queries: the roles of the ungrouped fused step; the table builders produce the
// tables of all G query heads from one pass over the key/value head's codebook.  Two workgroups per
// compute unit at group 2, one from group 4 on (as the unfused grouped kernel).
static size_t step_gqa_lds_bytes(int group, int m, int d_k)
{
    return gqa_lds_bytes(group, m, d_k, kStepWaves) + (size_t)m * kDecWaves * (sizeof(double) + sizeof(int));
}
template <int DK, typename FT, int G>
static int launch_step_gqa(const DecodeArgs &a, dim3 grid, hipStream_t st)
{
    dim3 block(kStepWaves * kWave);
    const size_t lds = step_gqa_lds_bytes(G, a.m, DK);
#define LOOKAT_STEP_GQA_CASE(M_)                                                                               \
    case M_: {                                                                                                 \
        auto kern = decode_split_kernel<DK, M_, kStepWaves, ((G == 2 && DK / M_ < 64) ? 4 : 2), FT, G, kStepPrefetch>; \
        if (lds > 64 * 1024) {                                                                                 \
            /* allow more than 64 KB of dynamic LDS: idempotent, so every call makes it (no shared flag) */   \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                          \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);         \
            if (e != hipSuccess)                                                                               \
                return fail(LOOKAT_ERR_HIP, "lookat_decode_step_gqa: cannot reserve %zu bytes of LDS: %s", lds, \
                            hipGetErrorString(e));                                                             \
        }                                                                                                      \
        hipLaunchKernelGGL(kern, grid, block, lds, st, LOOKAT_DECODE_HEAD_ARGS(a, true), late_of(a));          \
        return LOOKAT_OK;                                                                                      \
    }
    switch (a.m) {
        LOOKAT_STEP_GQA_CASE(2)
        LOOKAT_STEP_GQA_CASE(4)
        LOOKAT_STEP_GQA_CASE(8)
        LOOKAT_STEP_GQA_CASE(16)
    default:
        return fail(LOOKAT_ERR_UNSUPPORTED, "lookat_decode_step_gqa handles m in {2,4,8,16}; got m=%d", a.m);
    }
#undef LOOKAT_STEP_GQA_CASE
}

template <int DK, typename FT>
static int launch_step_gqa_group(int group, const DecodeArgs &a, dim3 grid, hipStream_t st)
{
    switch (group) {
    case 2:
        return launch_step_gqa<DK, FT, 2>(a, grid, st);
    case 4:
        return launch_step_gqa<DK, FT, 4>(a, grid, st);
    case 8:
        return launch_step_gqa<DK, FT, 8>(a, grid, st);
    default:
        return fail(LOOKAT_ERR_UNSUPPORTED, "lookat_decode_step_gqa handles group in {1,2,4,8}; got %d", group);
    }
}

template <int DK>
static int launch_gqa_dk(int group, const DecodeArgs &a, dim3 grid, hipStream_t st)
{
    switch (group) {
    case 2:
        return launch_gqa<DK, 2>(a, grid, st);
    case 4:
        return gqa_waves(4, a.m, DK) == kDecWaves ? launch_gqa<DK, 4>(a, grid, st)
                                                  : launch_gqa<DK, 4, 2 * kDecWaves>(a, grid, st);
    case 8:
        return gqa_waves(8, a.m, DK) == kDecWaves ? launch_gqa<DK, 8>(a, grid, st)
                                                  : launch_gqa<DK, 8, 2 * kDecWaves>(a, grid, st);
    default:
        return fail(LOOKAT_ERR_UNSUPPORTED, "lookat_attend_decode_gqa handles group in {1,2,4,8}; got %d", group);
    }
}

}  // namespace lookat

namespace lookat {
// Fused step, S ranges per (b,h) (S = 1: no workspace, results written directly).
// group > 1: shape->H counts key/value heads, q and out have group times as many heads.
static int decode_step_impl(const char *who, const lookat_shape *shape, int group, int64_t L, const void *q,
                            const void *k_new, int qk_dtype, const float *codebooks, uint8_t *codes,
                            int64_t code_stride_bh, const void *values, int64_t value_stride_bh, float scale, int S,
                            void *workspace, size_t workspace_bytes, float *out, void *stream, int force_entries = 0)
{
    // force_entries: 0 = the library's choice of batch entries per workgroup, 1 or 2 = that many (measurement aid).
    // (At d_k = 128 with m = 2 a codebook row alone is 64 registers: two entries' state does not fit the 128
    // registers of a 1024-thread workgroup, so there is no paired instance.)
    if (force_entries == 2 && (group != 1 || (shape->B & 1) || (shape->d_k != 64 && (shape->d_k != 128 || shape->m == 2))))
        return fail(LOOKAT_ERR_UNSUPPORTED,
                    "paired batch entries need an even batch, ungrouped queries and d_k = 64 or d_k = 128 with m > 2; "
                    "got B=%d group=%d d_k=%d m=%d", shape->B, group, shape->d_k, shape->m);
    const bool paired = force_entries == 2 || (force_entries == 0 && step_pairs_entries(shape, group, L, S));
    if (L <= 0)
        return fail(LOOKAT_ERR_SHAPE, "L=%lld must be positive", (long long)L);
    if (qk_dtype != LOOKAT_F16 && qk_dtype != LOOKAT_F32)
        return fail(LOOKAT_ERR_DTYPE, "qk_dtype=%d is neither LOOKAT_F16 nor LOOKAT_F32", qk_dtype);
    if (!q || !k_new || !codebooks || !codes || !values || !out)
        return fail(LOOKAT_ERR_NULL, "q, k_new, codebooks, codes, values and out must be non-NULL");
    if (code_stride_bh < L * shape->m || value_stride_bh < L * shape->d_k)
        return fail(LOOKAT_ERR_SHAPE, "code_stride_bh=%lld / value_stride_bh=%lld smaller than one (b,h) slab",
                    (long long)code_stride_bh, (long long)value_stride_bh);
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(codebooks) || !aligned16(values) || !aligned16(out) ||
        ((value_stride_bh * 2) % 16))
        return fail(LOOKAT_ERR_ALIGN, "q, k_new, codebooks, values, out and value_stride_bh must be 16-byte aligned");
    const bool m_ok = shape->m == 2 || shape->m == 4 || shape->m == 8 || shape->m == 16;
    if (!m_ok || (shape->d_k != 64 && shape->d_k != 128))
        return fail(LOOKAT_ERR_UNSUPPORTED,
                    "%s handles d_k in {64,128} with m in {2,4,8,16}; got d_k=%d m=%d "
                    "(use encode_keys + build_lut + attend_decode)", who, shape->d_k, shape->m);
    if ((reinterpret_cast<uintptr_t>(codes) % shape->m) || (code_stride_bh % shape->m))
        return fail(LOOKAT_ERR_ALIGN, "codes and code_stride_bh must be multiples of m=%d bytes", shape->m);
    if ((L + 2048) * (int64_t)shape->d_k * 2 > 0xffffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "L=%lld: one (b,h) value slab must stay below 4 GiB", (long long)L);
    if (code_stride_bh > 0xffffffffLL || value_stride_bh > 0xffffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "(b,h) strides must stay below 2^32 elements");
    if (group > 1 && step_gqa_lds_bytes(group, shape->m, shape->d_k) > 160 * 1024)
        return fail(LOOKAT_ERR_UNSUPPORTED, "group=%d x m=%d tables (%zu bytes with the reduction buffer) exceed the 160 KB of LDS",
                    group, shape->m, step_gqa_lds_bytes(group, shape->m, shape->d_k));
    const int64_t BH = (int64_t)shape->B * shape->H;
    const size_t need = (S == 1) ? 0 : (size_t)BH * group * S * (shape->d_k + 2) * sizeof(float);
    if (need) {
        if (!workspace || workspace_bytes < need)
            return fail(LOOKAT_ERR_WORKSPACE, "workspace of %zu bytes needed for %d splits, got %zu", need, S,
                        workspace_bytes);
        if (!aligned16(workspace))
            return fail(LOOKAT_ERR_ALIGN, "workspace must be 16-byte aligned");
    }
    const int64_t units = paired ? BH / 2 : BH;   // workgroups per range
    const int64_t nblocks = (units + kXcds - 1) / kXcds * kXcds * S;
    if (nblocks > 0x7fffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "B*H*num_splits=%lld workgroups exceed one launch", (long long)nblocks);

    DecodeArgs a;
    a.lut = nullptr;
    a.codes = codes;
    a.values = static_cast<const __half *>(values);
    a.part = static_cast<float *>(workspace);
    a.out = out;
    a.scores_out = nullptr;
    a.code_stride = code_stride_bh;
    a.value_stride = value_stride_bh;
    a.L = L;
    a.keys_per_split = round_up((L + S - 1) / S, kTile);
    a.BH = (int)BH;
    a.splits = S;
    a.d_k = shape->d_k;
    a.m = shape->m;
    a.scale_log2e = scale * kLog2e;
    a.q = q;
    a.k_new = k_new;
    a.codebooks = codebooks;
    a.codes_w = codes;
    a.H = shape->H;
    hipStream_t st = static_cast<hipStream_t>(stream);
    dim3 grid((unsigned)nblocks);
    if (group == 1) {
        bool ok;
        if (paired) {
            if (shape->d_k == 64)
                ok = (qk_dtype == LOOKAT_F16) ? launch_step_pair<64, __half>(a, grid, st)
                                              : launch_step_pair<64, float>(a, grid, st);
            else
                ok = (qk_dtype == LOOKAT_F16) ? launch_step_pair<128, __half>(a, grid, st)
                                              : launch_step_pair<128, float>(a, grid, st);
        } else if (shape->d_k == 64)
            ok = (qk_dtype == LOOKAT_F16) ? launch_step<64, __half>(a, grid, st) : launch_step<64, float>(a, grid, st);
        else
            ok = (qk_dtype == LOOKAT_F16) ? launch_step<128, __half>(a, grid, st) : launch_step<128, float>(a, grid, st);
        if (!ok)
            return fail(LOOKAT_ERR_UNSUPPORTED, "no fused kernel for this shape");
    } else {
        int rc;
        if (shape->d_k == 64)
            rc = (qk_dtype == LOOKAT_F16) ? launch_step_gqa_group<64, __half>(group, a, grid, st)
                                          : launch_step_gqa_group<64, float>(group, a, grid, st);
        else
            rc = (qk_dtype == LOOKAT_F16) ? launch_step_gqa_group<128, __half>(group, a, grid, st)
                                          : launch_step_gqa_group<128, float>(group, a, grid, st);
        if (rc != LOOKAT_OK)
            return rc;
    }
    if (S > 1)
        hipLaunchKernelGGL(decode_combine_kernel, dim3((unsigned)(BH * group)), dim3(kDecThreads), 0, st,
                           static_cast<const float *>(workspace), out, S, shape->d_k);
    return check_launch(who);
}
}  // namespace lookat

extern "C" int lookat_decode_step(const lookat_shape *shape, int64_t L, const void *q, const void *k_new,
                                  lookat_dtype qk_dtype, const float *codebooks, uint8_t *codes, int64_t code_stride_bh,
                                  const void *values, int64_t value_stride_bh, float scale, float *out, void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    return decode_step_impl("lookat_decode_step", shape, 1, L, q, k_new, qk_dtype, codebooks, codes, code_stride_bh, values,
                            value_stride_bh, scale, 1, nullptr, 0, out, stream);
}

extern "C" int32_t lookat_decode_step_entries_per_workgroup(const lookat_shape *shape, int64_t L)
{
    using namespace lookat;
    clear_error();
    if (check_shape(shape) != LOOKAT_OK || L <= 0)
        return 0;
    const bool m_ok = shape->m == 2 || shape->m == 4 || shape->m == 8 || shape->m == 16;
    if (!m_ok || (shape->d_k != 64 && shape->d_k != 128))
        return 0;
    return step_pairs_entries(shape, 1, L, 1) ? 2 : 1;
}

extern "C" int lookat_probe_decode_step_entries(const lookat_shape *shape, int32_t entries_per_workgroup, int64_t L,
                                                const void *q, const void *k_new, lookat_dtype qk_dtype,
                                                const float *codebooks, uint8_t *codes, int64_t code_stride_bh,
                                                const void *values, int64_t value_stride_bh, float scale, float *out,
                                                void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (entries_per_workgroup != 1 && entries_per_workgroup != 2)
        return fail(LOOKAT_ERR_SHAPE, "entries_per_workgroup=%d must be 1 or 2", entries_per_workgroup);
    return decode_step_impl("lookat_probe_decode_step_entries", shape, 1, L, q, k_new, qk_dtype, codebooks, codes,
                            code_stride_bh, values, value_stride_bh, scale, 1, nullptr, 0, out, stream,
                            entries_per_workgroup);
}

extern "C" size_t lookat_decode_step_split_workspace_bytes(const lookat_shape *shape, int64_t L, int32_t num_splits)
{
    return lookat_attend_decode_workspace_bytes(shape, L, num_splits);
}

extern "C" int lookat_decode_step_split(const lookat_shape *shape, int64_t L, const void *q, const void *k_new,
                                        lookat_dtype qk_dtype, const float *codebooks, uint8_t *codes, int64_t code_stride_bh,
                                        const void *values, int64_t value_stride_bh, float scale, int32_t num_splits,
                                        void *workspace, size_t workspace_bytes, float *out, void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (num_splits < 0 || num_splits > 65535)
        return fail(LOOKAT_ERR_SHAPE, "num_splits=%d out of range [0,65535]", num_splits);
    const int S = num_splits ? num_splits : (L > 0 ? auto_splits(shape, L) : 1);
    return decode_step_impl("lookat_decode_step_split", shape, 1, L, q, k_new, qk_dtype, codebooks, codes, code_stride_bh,
                            values, value_stride_bh, scale, S, workspace, workspace_bytes, out, stream);
}

extern "C" size_t lookat_decode_step_gqa_workspace_bytes(const lookat_shape *shape, int32_t group, int64_t L,
                                                         int32_t num_splits)
{
    return lookat_attend_decode_gqa_workspace_bytes(shape, group, L, num_splits);
}

extern "C" int lookat_decode_step_gqa(const lookat_shape *shape, int32_t group, int64_t L, const void *q,
                                      const void *k_new, lookat_dtype qk_dtype, const float *codebooks, uint8_t *codes,
                                      int64_t code_stride_bh, const void *values, int64_t value_stride_bh, float scale,
                                      int32_t num_splits, void *workspace, size_t workspace_bytes, float *out,
                                      void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (group != 1 && group != 2 && group != 4 && group != 8)
        return fail(LOOKAT_ERR_UNSUPPORTED, "lookat_decode_step_gqa handles group in {1,2,4,8}; got %d", group);
    if (num_splits < 0 || num_splits > 65535)
        return fail(LOOKAT_ERR_SHAPE, "num_splits=%d out of range [0,65535]", num_splits);
    const int S = num_splits ? num_splits
                             : (L > 0 ? (group == 1 ? auto_splits(shape, L) : auto_splits_gqa(shape, group, L)) : 1);
    return decode_step_impl("lookat_decode_step_gqa", shape, group, L, q, k_new, qk_dtype, codebooks, codes,
                            code_stride_bh, values, value_stride_bh, scale, S, workspace, workspace_bytes, out, stream);
}

extern "C" int32_t lookat_attend_decode_auto_splits(const lookat_shape *shape, int64_t L)
{
    using namespace lookat;
    clear_error();
    if (check_shape(shape) != LOOKAT_OK || L <= 0)
        return 0;
    return auto_splits(shape, L);
}

extern "C" int lookat_attend_decode_launch_shape(const lookat_shape *shape, int64_t L, int32_t num_splits,
                                                 int32_t *ranges, int32_t *wavefronts)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (L <= 0)
        return fail(LOOKAT_ERR_SHAPE, "L=%lld must be positive", (long long)L);
    if (num_splits < 0 || num_splits > 65535)
        return fail(LOOKAT_ERR_SHAPE, "num_splits=%d out of range [0,65535]", num_splits);
    const int S = num_splits ? num_splits : auto_splits(shape, L);
    if (ranges)
        *ranges = S;
    if (wavefronts)
        *wavefronts = tuned_dk(shape->d_k) ? pick_waves(shape->d_k, shape->m, round_up((L + S - 1) / S, kTile)) : kDecWaves;
    return LOOKAT_OK;
}

extern "C" size_t lookat_attend_decode_workspace_bytes(const lookat_shape *shape, int64_t L, int32_t num_splits)
{
    using namespace lookat;
    clear_error();
    if (check_shape(shape) != LOOKAT_OK || L <= 0 || num_splits < 0)
        return 0;
    const int S = num_splits ? num_splits : auto_splits(shape, L);
    if (S == 1)
        return 0;
    return (size_t)shape->B * shape->H * S * (shape->d_k + 2) * sizeof(float);
}

namespace lookat {
static int attend_decode_impl(const lookat_shape *shape, int64_t L, const float *lut, const uint8_t *codes,
                              int64_t code_stride_bh, const void *values, int64_t value_stride_bh, float scale,
                              int32_t num_splits, void *workspace, size_t workspace_bytes, float *out,
                              float *scores_out, void *stream)
{
    if (int rc = check_shape(shape))
        return rc;
    if (L <= 0)
        return fail(LOOKAT_ERR_SHAPE, "L=%lld must be positive", (long long)L);
    if (num_splits < 0 || num_splits > 65535)
        return fail(LOOKAT_ERR_SHAPE, "num_splits=%d out of range [0,65535]", num_splits);
    if (!lut || !codes || !values || !out)
        return fail(LOOKAT_ERR_NULL, "lut, codes, values and out must be non-NULL");
    if (code_stride_bh < L * shape->m || value_stride_bh < L * shape->d_k)
        return fail(LOOKAT_ERR_SHAPE, "code_stride_bh=%lld / value_stride_bh=%lld smaller than one (b,h) slab",
                    (long long)code_stride_bh, (long long)value_stride_bh);
    if (!aligned16(lut) || !aligned16(values) || !aligned16(out) || ((value_stride_bh * 2) % 16))
        return fail(LOOKAT_ERR_ALIGN, "lut, values, out and value_stride_bh must be 16-byte aligned");
    // a key's m codes are fetched with one m-byte load when m is 2, 4, 8 or 16
    const int cvec = (shape->m == 2 || shape->m == 4 || shape->m == 8 || shape->m == 16) ? shape->m : 1;
    if ((reinterpret_cast<uintptr_t>(codes) % cvec) || (code_stride_bh % cvec))
        return fail(LOOKAT_ERR_ALIGN, "codes and code_stride_bh must be multiples of %d bytes for m=%d", cvec,
                    shape->m);
    if (scores_out && (reinterpret_cast<uintptr_t>(scores_out) & 3u))
        return fail(LOOKAT_ERR_ALIGN, "scores_out must be 4-byte aligned");

    if (code_stride_bh > 0xffffffffLL || value_stride_bh > 0xffffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "(b,h) strides must stay below 2^32 elements");
    // kernels address one (b,h) slab with 32-bit byte offsets (plus one tile of prefetch)
    if ((L + 2048) * (int64_t)shape->d_k * 2 > 0xffffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "L=%lld: one (b,h) value slab must stay below 4 GiB", (long long)L);
    const int64_t BH = (int64_t)shape->B * shape->H;
    const int S = num_splits ? num_splits : auto_splits(shape, L);
    const size_t need = (S == 1) ? 0 : (size_t)BH * S * (shape->d_k + 2) * sizeof(float);
    if (need) {
        if (!workspace || workspace_bytes < need)
            return fail(LOOKAT_ERR_WORKSPACE, "workspace of %zu bytes needed for %d splits, got %zu", need, S,
                        workspace_bytes);
        if (!aligned16(workspace))
            return fail(LOOKAT_ERR_ALIGN, "workspace must be 16-byte aligned");
    }
    const int64_t groups = (BH + kXcds - 1) / kXcds;
    const int64_t nblocks = groups * kXcds * S;
    if (nblocks > 0x7fffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "B*H*num_splits=%lld workgroups exceed one launch", (long long)nblocks);

    DecodeArgs a;
    a.lut = lut;
    a.codes = codes;
    a.values = static_cast<const __half *>(values);
    a.part = static_cast<float *>(workspace);
    a.out = out;
    a.scores_out = scores_out;
    a.code_stride = code_stride_bh;
    a.value_stride = value_stride_bh;
    a.L = L;
    a.keys_per_split = round_up((L + S - 1) / S, kTile);
    a.BH = (int)BH;
    a.splits = S;
    a.d_k = shape->d_k;
    a.m = shape->m;
    a.scale_log2e = scale * kLog2e;
    a.q = nullptr;
    a.k_new = nullptr;
    a.codebooks = nullptr;
    a.codes_w = nullptr;
    a.H = shape->H;

    hipStream_t st = static_cast<hipStream_t>(stream);
    dim3 grid((unsigned)nblocks);
    if (tuned_dk(shape->d_k)) {
        const int waves = pick_waves(shape->d_k, shape->m, a.keys_per_split);
        switch (shape->d_k) {
        case 32:
            launch_tuned<32, 4, 4>(a, grid, st);
            break;
        case 64:
            if (waves == 16)
                launch_tuned<64, 16, 8>(a, grid, st);
            else
                launch_tuned<64, 4, 4>(a, grid, st);
            break;
        case 128:
            if (waves == 16)
                launch_tuned<128, 16, 8>(a, grid, st);
            else
                launch_tuned<128, 4, 4>(a, grid, st);
            break;
        default:
            launch_tuned<256, 4, 4>(a, grid, st);
            break;
        }
    } else {
        const size_t lds = ((size_t)shape->m * kCentroids + kDecThreads + kDecWaves) * sizeof(float);
        hipLaunchKernelGGL(decode_split_generic_kernel, grid, dim3(kDecThreads), lds, st, LOOKAT_DECODE_HEAD_ARGS(a, false),
                           late_of(a));
    }
    if (int rc = check_launch("lookat_attend_decode (split kernel)"))
        return rc;
    if (S > 1) {
        hipLaunchKernelGGL(decode_combine_kernel, dim3((unsigned)BH), dim3(kDecThreads), 0, st,
                           static_cast<const float *>(workspace), out, S, shape->d_k);
        return check_launch("lookat_attend_decode (combine kernel)");
    }
    return LOOKAT_OK;
}

// Scratch memory of lookat_attend_decode_noalloc: the per-range partial results, in the library's own
// device image instead of a caller's workspace.  Every GPU the library runs on holds one copy.
static __device__ __align__(256) float scratch[LOOKAT_NOALLOC_SCRATCH_BYTES / sizeof(float)];

// Device address of `scratch` on the current device (in host code the array's name is only a handle
// for this query), looked up once per device and kept.
static int scratch_address(float **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static float *known[kMaxDevices] = {};
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess || device < 0 || device >= kMaxDevices)
        return fail(LOOKAT_ERR_HIP, "lookat_attend_decode_noalloc: cannot identify the current device (%s, device %d)",
                    hipGetErrorString(e), device);
    std::lock_guard<std::mutex> hold(lock);
    if (!known[device]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(LOOKAT_ERR_HIP, "lookat_attend_decode_noalloc: hipGetSymbolAddress failed on device %d: %s", device,
                        hipGetErrorString(e));
        known[device] = static_cast<float *>(p);
    }
    *ptr = known[device];
    return LOOKAT_OK;
}
}  // namespace lookat

extern "C" int lookat_attend_decode(const lookat_shape *shape, int64_t L, const float *lut, const uint8_t *codes,
                                    int64_t code_stride_bh, const void *values, int64_t value_stride_bh, float scale,
                                    int32_t num_splits, void *workspace, size_t workspace_bytes, float *out,
                                    float *scores_out, void *stream)
{
    using namespace lookat;
    clear_error();
    return attend_decode_impl(shape, L, lut, codes, code_stride_bh, values, value_stride_bh, scale, num_splits, workspace,
                              workspace_bytes, out, scores_out, stream);
}

extern "C" int lookat_attend_decode_noalloc(const lookat_shape *shape, int64_t L, const float *lut, const uint8_t *codes,
                                            int64_t code_stride_bh, const void *values, int64_t value_stride_bh,
                                            float scale, int32_t num_splits, float *out, float *scores_out, void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (L <= 0)
        return fail(LOOKAT_ERR_SHAPE, "L=%lld must be positive", (long long)L);
    if (num_splits < 0 || num_splits > 65535)
        return fail(LOOKAT_ERR_SHAPE, "num_splits=%d out of range [0,65535]", num_splits);
    const size_t need = lookat_attend_decode_workspace_bytes(shape, L, num_splits);
    if (need > (size_t)LOOKAT_NOALLOC_SCRATCH_BYTES)
        return fail(LOOKAT_ERR_WORKSPACE,
                    "lookat_attend_decode_noalloc: B*H*ranges*(d_k+2) floats = %zu bytes exceed the library's %d bytes of "
                    "scratch memory; use lookat_attend_decode with a workspace", need, (int)LOOKAT_NOALLOC_SCRATCH_BYTES);
    float *ws = nullptr;
    if (need) {   // (one range per (b,h): no partial results, nothing to look up)
        if (int rc = scratch_address(&ws))
            return rc;
    }
    return attend_decode_impl(shape, L, lut, codes, code_stride_bh, values, value_stride_bh, scale, num_splits, ws,
                              need ? (size_t)LOOKAT_NOALLOC_SCRATCH_BYTES : 0, out, scores_out, stream);
}

extern "C" size_t lookat_attend_decode_gqa_workspace_bytes(const lookat_shape *shape, int32_t group, int64_t L,
                                                           int32_t num_splits)
{
    using namespace lookat;
    clear_error();
    if (check_shape(shape) != LOOKAT_OK || L <= 0 || num_splits < 0 || group < 1)
        return 0;
    const int S = num_splits ? num_splits : auto_splits_gqa(shape, group, L);
    if (S == 1)
        return 0;
    return (size_t)shape->B * shape->H * group * S * (shape->d_k + 2) * sizeof(float);
}

extern "C" int lookat_attend_decode_gqa(const lookat_shape *shape, int32_t group, int64_t L, const float *lut,
                                        const uint8_t *codes, int64_t code_stride_bh, const void *values,
                                        int64_t value_stride_bh, float scale, int32_t num_splits, void *workspace,
                                        size_t workspace_bytes, float *out, float *scores_out, void *stream)
{
    using namespace lookat;
    if (group == 1)
        return lookat_attend_decode(shape, L, lut, codes, code_stride_bh, values, value_stride_bh, scale, num_splits,
                                    workspace, workspace_bytes, out, scores_out, stream);
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (group != 2 && group != 4 && group != 8)
        return fail(LOOKAT_ERR_UNSUPPORTED, "group=%d: query heads per key/value head must be 1, 2, 4 or 8", group);
    if (L <= 0)
        return fail(LOOKAT_ERR_SHAPE, "L=%lld must be positive", (long long)L);
    if (num_splits < 0 || num_splits > 65535)
        return fail(LOOKAT_ERR_SHAPE, "num_splits=%d out of range [0,65535]", num_splits);
    if (!lut || !codes || !values || !out)
        return fail(LOOKAT_ERR_NULL, "lut, codes, values and out must be non-NULL");
    if (code_stride_bh < L * shape->m || value_stride_bh < L * shape->d_k)
        return fail(LOOKAT_ERR_SHAPE, "code_stride_bh=%lld / value_stride_bh=%lld smaller than one (b,h) slab",
                    (long long)code_stride_bh, (long long)value_stride_bh);
    if (!aligned16(lut) || !aligned16(values) || !aligned16(out) || ((value_stride_bh * 2) % 16))
        return fail(LOOKAT_ERR_ALIGN, "lut, values, out and value_stride_bh must be 16-byte aligned");
    const bool m_ok = shape->m == 2 || shape->m == 4 || shape->m == 8 || shape->m == 16;
    if (!m_ok || (shape->d_k != 64 && shape->d_k != 128))
        return fail(LOOKAT_ERR_UNSUPPORTED,
                    "lookat_attend_decode_gqa handles d_k in {64,128} with m in {2,4,8,16}; got d_k=%d m=%d", shape->d_k,
                    shape->m);
    if ((reinterpret_cast<uintptr_t>(codes) % shape->m) || (code_stride_bh % shape->m))
        return fail(LOOKAT_ERR_ALIGN, "codes and code_stride_bh must be multiples of m=%d bytes", shape->m);
    if (scores_out && (reinterpret_cast<uintptr_t>(scores_out) & 3u))
        return fail(LOOKAT_ERR_ALIGN, "scores_out must be 4-byte aligned");
    if (code_stride_bh > 0xffffffffLL || value_stride_bh > 0xffffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "(b,h) strides must stay below 2^32 elements");
    if ((L + 2048) * (int64_t)shape->d_k * 2 > 0xffffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "L=%lld: one (b,h) value slab must stay below 4 GiB", (long long)L);
    const size_t lds = gqa_lds_bytes(group, shape->m, shape->d_k, gqa_waves(group, shape->m, shape->d_k));
    if (lds > 160 * 1024)
        return fail(LOOKAT_ERR_UNSUPPORTED, "group=%d x m=%d tables (%zu bytes with the reduction buffer) exceed the 160 KB of LDS",
                    group, shape->m, lds);
    const int64_t BH = (int64_t)shape->B * shape->H;   // key/value heads
    const int S = num_splits ? num_splits : auto_splits_gqa(shape, group, L);
    const size_t need = (S == 1) ? 0 : (size_t)BH * group * S * (shape->d_k + 2) * sizeof(float);
    if (need) {
        if (!workspace || workspace_bytes < need)
            return fail(LOOKAT_ERR_WORKSPACE, "workspace of %zu bytes needed for %d splits, got %zu", need, S,
                        workspace_bytes);
        if (!aligned16(workspace))
            return fail(LOOKAT_ERR_ALIGN, "workspace must be 16-byte aligned");
    }
    const int64_t nblocks = (BH + kXcds - 1) / kXcds * kXcds * S;
    if (nblocks > 0x7fffffffLL || BH * group > 0x7fffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "B*H*num_splits=%lld workgroups exceed one launch", (long long)nblocks);

    DecodeArgs a;
    a.lut = lut;
    a.codes = codes;
    a.values = static_cast<const __half *>(values);
    a.part = static_cast<float *>(workspace);
    a.out = out;
    a.scores_out = scores_out;
    a.code_stride = code_stride_bh;
    a.value_stride = value_stride_bh;
    a.L = L;
    a.keys_per_split = round_up((L + S - 1) / S, kTile);
    a.BH = (int)BH;
    a.splits = S;
    a.d_k = shape->d_k;
    a.m = shape->m;
    a.scale_log2e = scale * kLog2e;
    a.q = nullptr;
    a.k_new = nullptr;
    a.codebooks = nullptr;
    a.codes_w = nullptr;
    a.H = shape->H;
    hipStream_t st = static_cast<hipStream_t>(stream);
    dim3 grid((unsigned)nblocks);
    const int rc = (shape->d_k == 64) ? launch_gqa_dk<64>(group, a, grid, st) : launch_gqa_dk<128>(group, a, grid, st);
    if (rc != LOOKAT_OK)
        return rc;
    if (int rc2 = check_launch("lookat_attend_decode_gqa (split kernel)"))
        return rc2;
    if (S > 1) {
        hipLaunchKernelGGL(decode_combine_kernel, dim3((unsigned)(BH * group)), dim3(kDecThreads), 0, st,
                           static_cast<const float *>(workspace), out, S, shape->d_k);
        return check_launch("lookat_attend_decode_gqa (combine kernel)");
    }
    return LOOKAT_OK;
}
