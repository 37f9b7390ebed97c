// Measurement aid: a plain streaming read of a buffer with 16-byte loads, eight in flight per lane.
// It moves the same bytes as a streaming-matmul launch and nothing else, so its duration is the
// practical floor (launch latency + memory pipeline) that the contraction kernels are judged against
// next to the 8 TB/s data-sheet figure.
#include "../../include/itq3s_bench.h"
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

constexpr int kProbeThreads = 512, kProbeUnroll = 8;

__global__ __launch_bounds__(kProbeThreads) void read_probe_kernel(const u32x4* __restrict__ p, size_t n16, uint32_t* __restrict__ sink) {
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;  // a contiguous slice per workgroup
    const size_t beg = per * blockIdx.x, end = beg + per < n16 ? beg + per : n16;
    u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = beg + threadIdx.x;
    for (; i + (kProbeUnroll - 1) * kProbeThreads < end; i += (size_t)kProbeUnroll * kProbeThreads) {
        u32x4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) v[u] = __builtin_nontemporal_load(p + i + (size_t)u * kProbeThreads);
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc |= v[u];
    }
    for (; i < end; i += kProbeThreads) acc |= __builtin_nontemporal_load(p + i);
    // a data-dependent store the compiler cannot drop; the value written depends on all bytes read
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9e3779b9u) sink[0] = x;
}

}  // namespace itq3s

extern "C" int itq3s_read_probe(const void* src, size_t bytes, uint32_t* sink, void* stream) {
    if (!src || !sink) return ITQ3S_ERR_NULL;
    if (bytes < 16) return ITQ3S_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 15) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3) != 0) return ITQ3S_ERR_ALIGN;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    const size_t n16 = bytes / 16;
    size_t grid = (n16 + itq3s::kProbeThreads - 1) / itq3s::kProbeThreads;
    if (grid > (size_t)cus * 2) grid = (size_t)cus * 2;
    hipLaunchKernelGGL(itq3s::read_probe_kernel, dim3((unsigned)grid), dim3(itq3s::kProbeThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const itq3s::u32x4*>(src), n16, sink);
    return hipGetLastError() == hipSuccess ? ITQ3S_OK : ITQ3S_ERR_LAUNCH;
}
