// Streaming-read probe: what HBM read bandwidth a plain kernel with this library's access pattern
// (16 bytes per lane, fully coalesced, several loads in flight per lane) reaches on the device.  It is a
// measuring aid for benchmarks, not a step of the method: the figures of the merge and attention
// kernels are quoted against the nominal peak, this probe says how much of that peak a kernel can get.
#include "sc_device.h"
#include "sc_host.h"

namespace sc {

constexpr int kProbeThreads = 768;
constexpr int kProbeUnroll = 8;
typedef unsigned int probe_u32x4_t __attribute__((ext_vector_type(4)));

// One workgroup of twelve wavefronts per CU, each streaming a contiguous slab of its own with eight loads of
// 16 bytes in flight per lane (96 KB per CU) and the non-temporal hint: the shape that read fastest of those
// tried on this device (7.1 TB/s; 2048 workgroups of 256 threads striding over the whole buffer: 5.4).
__global__ __launch_bounds__(kProbeThreads) void stream_read_kernel(const probe_u32x4_t *__restrict__ src, size_t n16, uint32_t *sink) {
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
    uint32_t acc = 0u;
    size_t i = lo + threadIdx.x;
    for (; i + (kProbeUnroll - 1) * kProbeThreads < hi; i += kProbeUnroll * kProbeThreads) {
        probe_u32x4_t v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * kProbeThreads);
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < hi; i += kProbeThreads) {
        const probe_u32x4_t v = __builtin_nontemporal_load(src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // keeps the loads alive; one word per wavefront
    acc ^= __shfl_xor(acc, 32, kWave);
    acc ^= __shfl_xor(acc, 16, kWave);
    acc ^= __shfl_xor(acc, 8, kWave);
    acc ^= __shfl_xor(acc, 4, kWave);
    acc ^= __shfl_xor(acc, 2, kWave);
    acc ^= __shfl_xor(acc, 1, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) sink[(blockIdx.x * (kProbeThreads / kWave) + threadIdx.x / kWave) & 1023] = acc;
}

hipError_t launch_stream_read_probe(const void *src, size_t bytes, void *sink, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hipLaunchKernelGGL(stream_read_kernel, dim3(cus > 0 ? cus : 256), dim3(kProbeThreads), 0, stream,
                       reinterpret_cast<const probe_u32x4_t *>(src), n16, reinterpret_cast<uint32_t *>(sink));
    return hipGetLastError();
}

}  // namespace sc
