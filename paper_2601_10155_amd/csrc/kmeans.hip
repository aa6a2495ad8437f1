// Codebook learning (paper Sec. 3.4, "Prototype Learning"): one Lloyd iteration of k-means
// per (head, subspace).  Assignment is the key encoder itself; the update moves every
// centroid to the mean of its members.  The mean is an fp64 sum taken in ascending key
// order by a single thread per (centroid, coordinate), so the result does not depend on
// scheduling and is reproducible bit for bit.
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
    dim3 grid((unsigned)((kCentroids * d_sub + kKmThreads - 1) / kKmThreads), (unsigned)shape->m, (unsigned)shape->H);
    hipLaunchKernelGGL(kmeans_update_kernel, grid, dim3(kKmThreads), 0, static_cast<hipStream_t>(stream), calib, assign,
                       codebooks_in, codebooks_out, Nc, shape->d_k, shape->m);
    return check_launch("lookat_kmeans_step (update kernel)");
}
