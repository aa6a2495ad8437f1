// Codebook learning (paper Sec. 3.4, "Prototype Learning"): one Lloyd iteration of k-means
// per (head, subspace).  Assignment is the key encoder itself; the update moves every
// centroid to the mean of its members.  The mean is an fp64 sum taken in ascending key
// order by a single thread per (centroid, coordinate), so the result does not depend on
// scheduling and is reproducible bit for bit.  Two kernels: member lists in LDS for
// calibration sets of up to kKmListMax keys per head, a plain scan of all keys beyond.
#include "common.h"

namespace lookat {

constexpr int kKmThreads = 256;

// thread e of (h, i) owns centroid c = e / d_sub, coordinate j = e % d_sub
//   grid = (ceil(256 * d_sub / 256), m, H)
__global__ __launch_bounds__(kKmThreads) void kmeans_update_kernel(const float *__restrict__ calib,
                                                                   const uint8_t *__restrict__ assign,
                                                                   const float *__restrict__ cb_in,
                                                                   float *__restrict__ cb_out, int64_t Nc, int d_k,
                                                                   int m)
{
    const int d_sub = d_k / m;
    const int i = blockIdx.y;
    const int h = blockIdx.z;
    const int e = blockIdx.x * kKmThreads + threadIdx.x;
    if (e >= kCentroids * d_sub)
        return;
    const int c = e / d_sub, j = e % d_sub;
    const uint8_t *as = assign + (int64_t)h * Nc * m + i;
    const float *x = calib + (int64_t)h * Nc * d_k + (int64_t)i * d_sub + j;
    double sum = 0.0;
    int64_t cnt = 0;
    for (int64_t n = 0; n < Nc; ++n) {
        if (as[n * m] == c) {
            sum += (double)x[n * d_k];
            ++cnt;
        }
    }
    const int64_t o = (((int64_t)h * m + i) * kCentroids + c) * d_sub + j;
    cb_out[o] = cnt ? (float)(sum / (double)cnt) : cb_in[o];   // a centroid without members stays
}

// The same update for calibration sets that fit LDS (Nc <= kKmListMax): one workgroup per (h, i)
// first turns the assignment column into per-centroid member lists, then thread (c, j) adds only
// the members of c.  The lists hold the members in ascending key order, so every sum is taken in
// the order the scan above takes it and the result is the same bit for bit, at Nc / 256 loads per
// thread on average instead of Nc.
// List building is a stable counting sort by code.  Each of the four wavefronts owns a contiguous
// quarter of the keys: it histograms its quarter (LDS atomics; counts do not depend on order),
// the 256 threads turn the four histograms into every (wavefront, code) pair's first slot, and
// each wavefront then walks its quarter 64 keys at a time in ascending order: the lanes that hold
// equal codes find each other with eight ballots (one per code bit), a lane's slot is the pair's
// running offset plus the number of equal-code lanes below it, and the lowest of them advances
// the offset.  (LDS operations of one wavefront execute in program order.)
//   LDS: codes [Nc rounded up to 16] bytes | first[257] | run[4][256] | list [Nc] uint16
//   grid = (m, H), 256 threads
constexpr int kKmListMax = 16384;
constexpr int kKmWaves = kKmThreads / kWave;
static_assert(kKmThreads == kCentroids, "thread c owns the offsets of centroid c");

__host__ __device__ inline size_t km_codes_bytes(int64_t Nc) { return (size_t)((Nc + 15) / 16 * 16); }
__host__ __device__ inline size_t km_lds_bytes(int64_t Nc)
{
    return km_codes_bytes(Nc) + (kCentroids + 1 + kKmWaves * kCentroids) * sizeof(uint32_t) + (size_t)Nc * sizeof(uint16_t);
}

__global__ __launch_bounds__(kKmThreads) void kmeans_update_lists_kernel(const float *__restrict__ calib,
                                                                         const uint8_t *__restrict__ assign,
                                                                         const float *__restrict__ cb_in,
                                                                         float *__restrict__ cb_out, int Nc, int d_k,
                                                                         int m)
{
    extern __shared__ __align__(16) unsigned char km_smem[];
    uint8_t *codes_s = km_smem;
    uint32_t *first_s = reinterpret_cast<uint32_t *>(km_smem + km_codes_bytes(Nc));   // [257]
    uint32_t *run_s = first_s + kCentroids + 1;                                         // [waves][256]
    uint16_t *list_s = reinterpret_cast<uint16_t *>(run_s + kKmWaves * kCentroids);     // [Nc]
    __shared__ uint32_t wave_tot[kKmWaves];

    const int d_sub = d_k / m;
    const int i = blockIdx.x;
    const int h = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const uint8_t *as = assign + (int64_t)h * Nc * m + i;

    for (int n = tid; n < Nc; n += kKmThreads)
        codes_s[n] = as[(int64_t)n * m];
#pragma unroll
    for (int w = 0; w < kKmWaves; ++w)
        run_s[w * kCentroids + tid] = 0u;
    __syncthreads();

    // this wavefront's quarter of the keys: [q0, q1), a multiple of 64 long except at the end
    const int per = ((Nc + kKmWaves * kWave - 1) / (kKmWaves * kWave)) * kWave;
    const int q0 = wave * per < Nc ? wave * per : Nc;
    const int q1 = q0 + per < Nc ? q0 + per : Nc;
    uint32_t *run_w = run_s + wave * kCentroids;
    for (int n = q0 + lane; n < q1; n += kWave)
        atomicAdd(&run_w[codes_s[n]], 1u);
    __syncthreads();

    // thread c: members of c per wavefront -> first slot of (wavefront, c); exclusive prefix sum over c
    uint32_t hw[kKmWaves], cnt = 0;
#pragma unroll
    for (int w = 0; w < kKmWaves; ++w) {
        hw[w] = run_s[w * kCentroids + tid];
        cnt += hw[w];
    }
    uint32_t incl = cnt;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d);
        if (lane >= d)
            incl += up;
    }
    if (lane == kWave - 1)
        wave_tot[wave] = incl;
    __syncthreads();
    uint32_t pos = incl - cnt;
    for (int w = 0; w < wave; ++w)
        pos += wave_tot[w];
    first_s[tid] = pos;
    if (tid == kKmThreads - 1)
        first_s[kCentroids] = pos + cnt;
#pragma unroll
    for (int w = 0; w < kKmWaves; ++w) {
        run_s[w * kCentroids + tid] = pos;
        pos += hw[w];
    }
    __syncthreads();

    for (int n0 = q0; n0 < q1; n0 += kWave) {   // wave-uniform trip count
        const int n = n0 + lane;
        const bool valid = n < q1;
        const uint32_t code = valid ? codes_s[n] : 0u;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const uint64_t set = __ballot((code >> bit) & 1u);
            peers &= ((code >> bit) & 1u) ? set : ~set;
        }
        const uint32_t below = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        const uint32_t slot = run_w[code];
        if (valid)
            list_s[slot + below] = (uint16_t)n;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();   // every lane has read the offset before it moves
        if (valid && below == 0)
            run_w[code] = slot + (uint32_t)__popcll(peers);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();

    const float *x0 = calib + (int64_t)h * Nc * d_k + (int64_t)i * d_sub;
    for (int e = tid; e < kCentroids * d_sub; e += kKmThreads) {
        const int c = e / d_sub, j = e % d_sub;
        const uint32_t f = first_s[c], l = first_s[c + 1];
        const float *x = x0 + j;
        double sum = 0.0;
        uint32_t u = f;
        for (; u + 4 <= l; u += 4) {   // four loads in flight, added in list order
            const float a0 = x[(int64_t)list_s[u] * d_k], a1 = x[(int64_t)list_s[u + 1] * d_k];
            const float a2 = x[(int64_t)list_s[u + 2] * d_k], a3 = x[(int64_t)list_s[u + 3] * d_k];
            sum += (double)a0;
            sum += (double)a1;
            sum += (double)a2;
            sum += (double)a3;
        }
        for (; u < l; ++u)
            sum += (double)x[(int64_t)list_s[u] * d_k];
        const int64_t o = (((int64_t)h * m + i) * kCentroids + c) * d_sub + j;
        cb_out[o] = (l > f) ? (float)(sum / (double)(int64_t)(l - f)) : cb_in[o];   // a centroid without members stays
    }
}

}  // namespace lookat

extern "C" int lookat_kmeans_step(const lookat_shape *shape, int64_t Nc, const float *calib,
                                  const float *codebooks_in, float *codebooks_out, uint8_t *assign, void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (shape->B != 1)
        return fail(LOOKAT_ERR_SHAPE, "kmeans_step takes one calibration set per head: B must be 1, got %d", shape->B);
    if (Nc <= 0)
        return fail(LOOKAT_ERR_SHAPE, "Nc=%lld must be positive", (long long)Nc);
    if (!calib || !codebooks_in || !codebooks_out || !assign)
        return fail(LOOKAT_ERR_NULL, "calib, codebooks_in, codebooks_out and assign must be non-NULL");
    if (codebooks_in == codebooks_out)
        return fail(LOOKAT_ERR_SHAPE, "codebooks_out must not alias codebooks_in");
    if (int rc = lookat_encode_keys(shape, Nc, calib, LOOKAT_F32, codebooks_in, assign, Nc * shape->m, stream))
        return rc;
    const int d_sub = shape->d_k / shape->m;
    if (Nc <= kKmListMax) {
        const size_t lds = km_lds_bytes(Nc);
        hipLaunchKernelGGL(kmeans_update_lists_kernel, dim3((unsigned)shape->m, (unsigned)shape->H), dim3(kKmThreads), lds,
                           static_cast<hipStream_t>(stream), calib, assign, codebooks_in, codebooks_out, (int)Nc, shape->d_k,
                           shape->m);
        return check_launch("lookat_kmeans_step (update kernel, member lists)");
    }
    dim3 grid((unsigned)((kCentroids * d_sub + kKmThreads - 1) / kKmThreads), (unsigned)shape->m, (unsigned)shape->H);
    hipLaunchKernelGGL(kmeans_update_kernel, grid, dim3(kKmThreads), 0, static_cast<hipStream_t>(stream), calib, assign,
                       codebooks_in, codebooks_out, Nc, shape->d_k, shape->m);
    return check_launch("lookat_kmeans_step (update kernel)");
}
