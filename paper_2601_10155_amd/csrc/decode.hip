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
#include "common.h"

namespace lookat {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWave;
constexpr int kTile = 64;          // keys per wavefront tile: one key per lane in the score phase
constexpr int kXcds = 8;           // accelerator dies; workgroup ids are dealt round-robin to them
constexpr float kLog2e = 1.4426950408889634f;

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
};

// Workgroup id -> (bh, split).  Consecutive workgroup ids land on different dies, each
// with its own L2; this mapping keeps all splits of one (b,h) on one die so that its
// table is fetched into a single L2.
__device__ __forceinline__ bool map_block(const DecodeArgs &a, int &bh, int &split)
{
    const int bid = blockIdx.x;
    const int xcd = bid % kXcds;
    const int slot = bid / kXcds;
    bh = (slot / a.splits) * kXcds + xcd;
    split = slot % a.splits;
    return bh < a.BH;
}

template <int M>
struct CodeLoad;
template <>
struct CodeLoad<2> {
    using type = uint16_t;
};
template <>
struct CodeLoad<4> {
    using type = uint32_t;
};
template <>
struct CodeLoad<8> {
    using type = uint2;
};
template <>
struct CodeLoad<16> {
    using type = uint4;
};

__device__ __forceinline__ uint32_t code_word(const uint16_t &c, int) { return c; }
__device__ __forceinline__ uint32_t code_word(const uint32_t &c, int) { return c; }
__device__ __forceinline__ uint32_t code_word(const uint2 &c, int w) { return w == 0 ? c.x : c.y; }
__device__ __forceinline__ uint32_t code_word(const uint4 &c, int w)
{
    return w == 0 ? c.x : (w == 1 ? c.y : (w == 2 ? c.z : c.w));
}

// Unscaled ADC score of one key.  M > 0: the key's m codes are loaded as one vector.
template <int M>
__device__ __forceinline__ float adc_score(const float *lut_s, const uint8_t *code_ptr, int /*m*/)
{
    using CT = typename CodeLoad<M>::type;
    const CT c = *reinterpret_cast<const CT *>(code_ptr);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < M; ++i) {
        const uint32_t byte = (code_word(c, i / 4) >> (8 * (i % 4))) & 0xffu;
        s += lut_s[i * kCentroids + byte];
    }
    return s;
}
template <>
__device__ __forceinline__ float adc_score<0>(const float *lut_s, const uint8_t *code_ptr, int m)
{
    float s = 0.f;
    for (int i = 0; i < m; ++i)
        s += lut_s[i * kCentroids + code_ptr[i]];
    return s;
}

__device__ __forceinline__ void fma_row(float (&acc)[8], float p, const uint4 &v)
{
    const __half2 *h = reinterpret_cast<const __half2 *>(&v);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float2 f = __half22float2(h[k]);
        acc[2 * k] = fmaf(p, f.x, acc[2 * k]);
        acc[2 * k + 1] = fmaf(p, f.y, acc[2 * k + 1]);
    }
}

// Loads CH consecutive wave-wide row groups of a tile, starting at group g0; rows past the
// end of the range read as zero.
template <int DK, int CH>
__device__ __forceinline__ void load_rows(uint4 (&v)[CH], const __half *values_bh, int64_t kb, int64_t k1, int g0,
                                          int rowin, int sub)
{
    constexpr int RPL = kWave / (DK / 8);
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int64_t row = kb + (g0 + j) * RPL + rowin;
        v[j] = make_uint4(0u, 0u, 0u, 0u);
        if (row < k1)
            v[j] = *reinterpret_cast<const uint4 *>(values_bh + row * DK + sub * 8);
    }
}

// DK in {32, 64, 128, 256}; M in {2, 4, 8, 16} or 0 (= runtime m, byte loads).
template <int DK, int M>
__global__ __launch_bounds__(kDecThreads) void decode_split_kernel(const DecodeArgs a)
{
    constexpr int LPR = DK / 8;            // lanes per value row (16 bytes per lane)
    constexpr int RPL = kWave / LPR;       // value rows covered by one wave-wide load
    constexpr int NLD = kTile / RPL;       // wave-wide loads per tile (= LPR)
    constexpr int CH = NLD < 8 ? NLD : 8;  // loads kept in flight together

    extern __shared__ __align__(16) float smem[];
    float *lut_s = smem;                                   // [m][256]
    float *red_s = smem + (M ? M : a.m) * kCentroids;      // [kDecWaves][DK + 2]

    int bh, split;
    if (!map_block(a, bh, split))
        return;
    const int m = M ? M : a.m;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;

    {   // stage the table of this (b,h): m KB, 16 bytes per thread per step
        const float4 *g = reinterpret_cast<const float4 *>(a.lut + (int64_t)bh * m * kCentroids);
        float4 *s4 = reinterpret_cast<float4 *>(lut_s);
        for (int x = tid; x < m * (kCentroids / 4); x += kDecThreads)
            s4[x] = g[x];
    }
    __syncthreads();

    const int64_t k0 = (int64_t)split * a.keys_per_split;
    const int64_t k1 = (k0 + a.keys_per_split < a.L) ? (k0 + a.keys_per_split) : a.L;
    const uint8_t *codes_bh = a.codes + (int64_t)bh * a.code_stride;
    const __half *values_bh = a.values + (int64_t)bh * a.value_stride;
    const int sub = lane % LPR;      // which 8-coordinate slice of the value row
    const int rowin = lane / LPR;    // which row of a wave-wide load

    float m_run = -INFINITY;         // running max of scale*log2e*s over this wave's keys
    float z = 0.f;                   // per-lane share of the running sum
    float acc[8];
#pragma unroll
    for (int d = 0; d < 8; ++d)
        acc[d] = 0.f;

    for (int64_t kb = k0 + (int64_t)wave * kTile; kb < k1; kb += (int64_t)kDecWaves * kTile) {
        // value rows of the tile: LPR lanes per row, RPL rows per wave-wide load.  The first
        // group of loads is issued before the score phase so that its latency is covered.
        uint4 v[CH];
        load_rows<DK, CH>(v, values_bh, kb, k1, 0, rowin, sub);

        // ---- score phase: lane = key ----
        const int64_t key = kb + lane;
        float s = -INFINITY;
        if (key < k1) {
            const float raw = adc_score<M>(lut_s, codes_bh + key * m, m);
            if (a.scores_out)
                a.scores_out[(int64_t)bh * a.L + key] = raw;
            s = raw * a.scale_log2e;
        }
        const float m_new = fmaxf(m_run, wave_max(s));
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = fast_exp2(m_run - m_use);
        const float p = fast_exp2(s - m_use);
        z = z * corr + p;
#pragma unroll
        for (int d = 0; d < 8; ++d)
            acc[d] *= corr;
        m_run = m_new;

        // ---- value phase ----
#pragma unroll
        for (int c0 = 0; c0 < NLD; c0 += CH) {
            uint4 w[CH];
#pragma unroll
            for (int j = 0; j < CH; ++j)
                w[j] = v[j];
            if (c0 + CH < NLD)
                load_rows<DK, CH>(v, values_bh, kb, k1, c0 + CH, rowin, sub);
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                const float pj = __shfl(p, (c0 + j) * RPL + rowin);
                fma_row(acc, pj, w[j]);
            }
        }
    }

    // ---- fold the rows of the wave, then the waves of the workgroup ----
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
        for (int d = 0; d < 8; ++d)
            acc[d] += __shfl_xor(acc[d], off);
    }
    z = wave_sum(z);
    float *mine = red_s + wave * (DK + 2);
    if (lane < LPR) {
#pragma unroll
        for (int d = 0; d < 8; ++d)
            mine[sub * 8 + d] = acc[d];
    }
    if (lane == 0) {
        mine[DK] = m_run;
        mine[DK + 1] = z;
    }
    __syncthreads();

    if (tid < DK) {
        float mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w)
            mx = fmaxf(mx, red_s[w * (DK + 2) + DK]);
        const float m_use = (mx == -INFINITY) ? 0.f : mx;
        float o = 0.f, zz = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) {
            const float wgt = fast_exp2(red_s[w * (DK + 2) + DK] - m_use);
            o = fmaf(wgt, red_s[w * (DK + 2) + tid], o);
            zz = fmaf(wgt, red_s[w * (DK + 2) + DK + 1], zz);
        }
        if (a.splits == 1) {
            a.out[(int64_t)bh * DK + tid] = o / zz;
        } else {
            float *dst = a.part + ((int64_t)bh * a.splits + split) * (DK + 2);
            dst[tid] = o;
            if (tid == 0) {
                dst[DK] = mx;
                dst[DK + 1] = zz;
            }
        }
    }
}

// Any d_k (multiple of 8, <= 256) and any m: one 256-key tile per step, scores through LDS,
// thread j owns output coordinate j.  Used for head dimensions without a tuned kernel.
__global__ __launch_bounds__(kDecThreads) void decode_split_generic_kernel(const DecodeArgs a)
{
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
            const float raw = adc_score<0>(lut_s, codes_bh + key * m, m);
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
//   grid = BH, block = 256 (threads >= d_k idle)
__global__ __launch_bounds__(kDecThreads) void decode_combine_kernel(const float *__restrict__ part,
                                                                     float *__restrict__ out, int splits, int d_k)
{
    const int bh = blockIdx.x;
    const int tid = threadIdx.x;
    if (tid >= d_k)
        return;
    const float *p = part + (int64_t)bh * splits * (d_k + 2);
    float mx = -INFINITY;
    for (int s = 0; s < splits; ++s)
        mx = fmaxf(mx, p[s * (d_k + 2) + d_k]);
    const float m_use = (mx == -INFINITY) ? 0.f : mx;
    float o = 0.f, z = 0.f;
    for (int s = 0; s < splits; ++s) {
        const float w = fast_exp2(p[s * (d_k + 2) + d_k] - m_use);
        o = fmaf(w, p[s * (d_k + 2) + tid], o);
        z = fmaf(w, p[s * (d_k + 2) + d_k + 1], z);
    }
    out[(int64_t)bh * d_k + tid] = o / z;
}

static int64_t round_up(int64_t x, int64_t q) { return (x + q - 1) / q * q; }

static int auto_splits(const lookat_shape *s, int64_t L)
{
    // aim at >= ~4 workgroups per compute unit, but never ranges shorter than one
    // 64-key tile per wavefront
    const int64_t BH = (int64_t)s->B * s->H;
    int64_t want = (1024 + BH - 1) / BH;
    int64_t cap = (L + kDecWaves * kTile - 1) / (kDecWaves * kTile);
    if (want > cap)
        want = cap;
    if (want < 1)
        want = 1;
    if (want > 256)
        want = 256;
    return (int)want;
}

static bool tuned_dk(int d_k) { return d_k == 32 || d_k == 64 || d_k == 128 || d_k == 256; }

template <int DK>
static void launch_tuned(const DecodeArgs &a, dim3 grid, size_t lds, hipStream_t st)
{
    dim3 block(kDecThreads);
    switch (a.m) {
    case 2:
        hipLaunchKernelGGL((decode_split_kernel<DK, 2>), grid, block, lds, st, a);
        break;
    case 4:
        hipLaunchKernelGGL((decode_split_kernel<DK, 4>), grid, block, lds, st, a);
        break;
    case 8:
        hipLaunchKernelGGL((decode_split_kernel<DK, 8>), grid, block, lds, st, a);
        break;
    case 16:
        hipLaunchKernelGGL((decode_split_kernel<DK, 16>), grid, block, lds, st, a);
        break;
    default:
        hipLaunchKernelGGL((decode_split_kernel<DK, 0>), grid, block, lds, st, a);
        break;
    }
}

}  // namespace lookat

extern "C" int32_t lookat_attend_decode_auto_splits(const lookat_shape *shape, int64_t L)
{
    using namespace lookat;
    clear_error();
    if (check_shape(shape) != LOOKAT_OK || L <= 0)
        return 0;
    return auto_splits(shape, L);
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

extern "C" int lookat_attend_decode(const lookat_shape *shape, int64_t L, const float *lut, const uint8_t *codes,
                                    int64_t code_stride_bh, const void *values, int64_t value_stride_bh, float scale,
                                    int32_t num_splits, void *workspace, size_t workspace_bytes, float *out,
                                    float *scores_out, void *stream)
{
    using namespace lookat;
    clear_error();
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

    hipStream_t st = static_cast<hipStream_t>(stream);
    dim3 grid((unsigned)nblocks);
    if (tuned_dk(shape->d_k)) {
        const size_t lds = ((size_t)shape->m * kCentroids + (size_t)kDecWaves * (shape->d_k + 2)) * sizeof(float);
        switch (shape->d_k) {
        case 32:
            launch_tuned<32>(a, grid, lds, st);
            break;
        case 64:
            launch_tuned<64>(a, grid, lds, st);
            break;
        case 128:
            launch_tuned<128>(a, grid, lds, st);
            break;
        default:
            launch_tuned<256>(a, grid, lds, st);
            break;
        }
    } else {
        const size_t lds = ((size_t)shape->m * kCentroids + kDecThreads + kDecWaves) * sizeof(float);
        hipLaunchKernelGGL(decode_split_generic_kernel, grid, dim3(kDecThreads), lds, st, a);
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
