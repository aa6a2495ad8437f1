// Plain read-stream and write-stream kernels used to measure what the HBM paths deliver on the
// buffers the kernels stream (ceilings for their bandwidth figures, not part of the method).
#include "common.h"
#include "lookat_probe.h"

namespace lookat {

constexpr int kProbeThreads = 256;
constexpr int kProbeLoads = 2;   // 16-byte loads per thread; small workgroups stream best on MI355X
constexpr int kProbeStores = 1;  // 16-byte stores per thread: 4 KB per workgroup wrote fastest (6.9 TB/s over 4 GB; 6.1 with two, 5.7 with eight)

typedef unsigned int probe_v4u __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kProbeThreads) void stream_read_kernel(const uint4 *__restrict__ p, size_t n16,
                                                                    uint32_t *sink)
{
    const probe_v4u *pv = reinterpret_cast<const probe_v4u *>(p);
    const size_t base = (size_t)blockIdx.x * (kProbeLoads * kProbeThreads) + threadIdx.x;
    uint4 v[kProbeLoads];
#pragma unroll
    for (int j = 0; j < kProbeLoads; ++j) {
        const size_t i = base + (size_t)j * kProbeThreads;
        // non-temporal: read once (6.06 against 5.70 TB/s on 48 MB buffers)
        const probe_v4u t = (i < n16) ? __builtin_nontemporal_load(pv + i) : probe_v4u{0u, 0u, 0u, 0u};
        v[j] = make_uint4(t.x, t.y, t.z, t.w);
    }
    uint32_t x = 0;
#pragma unroll
    for (int j = 0; j < kProbeLoads; ++j)
        x ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    if (x == 0x9e3779b9u && v[0].y == 0x7f4a7c15u && v[0].z == 0xf39cc060u)
        sink[0] = x;
}

__global__ __launch_bounds__(kProbeThreads) void stream_write_kernel(uint4 *__restrict__ p, size_t n16, uint32_t word)
{
    const size_t base = (size_t)blockIdx.x * (kProbeStores * kProbeThreads) + threadIdx.x;
    const uint4 v = make_uint4(word, word, word, word);
#pragma unroll
    for (int j = 0; j < kProbeStores; ++j) {
        const size_t i = base + (size_t)j * kProbeThreads;
        if (i < n16)
            p[i] = v;
    }
}

}  // namespace lookat

extern "C" int lookat_probe_stream_write(void *dst, size_t bytes, uint32_t word, void *stream)
{
    using namespace lookat;
    clear_error();
    if (!dst)
        return fail(LOOKAT_ERR_NULL, "dst must be non-NULL");
    if (bytes == 0 || (bytes % 16))
        return fail(LOOKAT_ERR_SHAPE, "bytes=%zu must be a positive multiple of 16", bytes);
    if (!aligned16(dst))
        return fail(LOOKAT_ERR_ALIGN, "dst must be 16-byte aligned");
    const size_t n16 = bytes / 16;
    const size_t per_block = (size_t)kProbeStores * kProbeThreads;
    const size_t blocks = (n16 + per_block - 1) / per_block;
    if (blocks > 0x7fffffffULL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "bytes=%zu exceed one launch", bytes);
    hipLaunchKernelGGL(stream_write_kernel, dim3((unsigned)blocks), dim3(kProbeThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<uint4 *>(dst), n16, word);
    return check_launch("lookat_probe_stream_write");
}

extern "C" int lookat_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    using namespace lookat;
    clear_error();
    if (!src || !sink)
        return fail(LOOKAT_ERR_NULL, "src and sink must be non-NULL");
    if (bytes == 0 || (bytes % 16))
        return fail(LOOKAT_ERR_SHAPE, "bytes=%zu must be a positive multiple of 16", bytes);
    if (!aligned16(src))
        return fail(LOOKAT_ERR_ALIGN, "src must be 16-byte aligned");
    const size_t n16 = bytes / 16;
    const size_t per_block = (size_t)kProbeLoads * kProbeThreads;
    const size_t blocks = (n16 + per_block - 1) / per_block;
    if (blocks > 0x7fffffffULL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "bytes=%zu exceed one launch", bytes);
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(kProbeThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint4 *>(src), n16, sink);
    return check_launch("lookat_probe_stream_read");
}
