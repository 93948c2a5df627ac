// What a plain streaming read achieves on this GPU: the context figure beside the vendor's peak that the
// list scan's bandwidth is quoted against (the paper's Sec. 2 roofline takes the memory bandwidth as given).
// Grid-stride reads of 16 bytes per lane, U in flight per lane, nothing else; the best of a few launch shapes
// (U = 8 or 16 loads in flight, 4, 8 or 16 workgroups per compute unit, plain or non-temporal loads) is reported.
#include "../../include/trinity_ivf.h"
#include "tri_common.h"

#include <algorithm>

namespace {

typedef unsigned int probe_u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ uint4 probe_ld(const uint4 *p)
{
    if (!NT) return *p;
    const probe_u32x4 v = __builtin_nontemporal_load((const probe_u32x4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <int U, bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ p, size_t n16, uint32_t *__restrict__ sink)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    size_t i = tid;
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = probe_ld<NT>(p + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n16; i += stride) { const uint4 v = probe_ld<NT>(p + i); acc ^= v.x ^ v.y ^ v.z ^ v.w; }
    if (acc == 0x9E3779B9u) sink[0] = acc;         // (keeps the loads alive; practically never taken)
}

}  // namespace

extern "C" int tri_stream_read_bandwidth(const void *dev_buf, size_t bytes, void *dev_sink, void *hip_stream, uint32_t repeats,
                                         double *gb_per_s)
{
    if (!dev_buf || !dev_sink || !gb_per_s || bytes < (1u << 20) || repeats == 0 || (uintptr_t)dev_buf % 16)
        return tri_fail(TRI_EINVAL, "need a 16-byte aligned device buffer of at least 1 MiB, a 4-byte device sink, repeats >= 1");
    hipStream_t s = (hipStream_t)hip_stream;
    int dev = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    hipEvent_t a = nullptr, b = nullptr;
    if (e == hipSuccess) e = hipEventCreate(&a);
    if (e == hipSuccess) e = hipEventCreate(&b);
    const size_t n16 = bytes / 16;
    const dim3 block(256);
    double best = 0.0;
    for (int shape = 0; shape < 12 && e == hipSuccess; ++shape) {
        const dim3 grid((unsigned)prop.multiProcessorCount * (4u << (shape % 3)));
        const bool wide = shape % 6 >= 3, nt = shape >= 6;
        auto launch = [&]() {
            if (wide && nt) hipLaunchKernelGGL((stream_read_kernel<16, true>), grid, block, 0, s, (const uint4 *)dev_buf, n16, (uint32_t *)dev_sink);
            else if (wide) hipLaunchKernelGGL((stream_read_kernel<16, false>), grid, block, 0, s, (const uint4 *)dev_buf, n16, (uint32_t *)dev_sink);
            else if (nt) hipLaunchKernelGGL((stream_read_kernel<8, true>), grid, block, 0, s, (const uint4 *)dev_buf, n16, (uint32_t *)dev_sink);
            else hipLaunchKernelGGL((stream_read_kernel<8, false>), grid, block, 0, s, (const uint4 *)dev_buf, n16, (uint32_t *)dev_sink);
        };
        float ms = 0.f;
        launch();                                                   // warm-up
        e = hipEventRecord(a, s);
        for (uint32_t r = 0; r < repeats && e == hipSuccess; ++r) {
            launch();
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipEventRecord(b, s);
        if (e == hipSuccess) e = hipEventSynchronize(b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
        if (e == hipSuccess && ms > 0.f) best = std::max(best, (double)(n16 * 16) * repeats / (ms * 1e-3) / 1e9);
    }
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    if (e != hipSuccess) return tri_fail(TRI_EHIP, "streaming-read probe -> %s", hipGetErrorString(e));
    *gb_per_s = best;
    return TRI_OK;
}
