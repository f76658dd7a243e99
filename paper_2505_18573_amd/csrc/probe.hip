// Read-bandwidth probe for gfx950: streams a device buffer once with the access pattern
// of the vocabulary pass (16-byte non-temporal loads, a wave instruction covering 1 KiB
// of contiguous memory, eight loads in flight per lane) and does nothing else but fold
// the data into per-workgroup xor checksums.  It contains no arithmetic of the method;
// the benchmark times it on its own logit buffers so that the kernels' achieved GB/s can
// be read against what a pure read of the same bytes reaches on the same machine.
#include "vocab_common.h"
#include "vocab_pass.h"
#include <hip/hip_ext.h>

namespace e3 {
namespace {

constexpr int kProbeThreads = 256;

__global__ __launch_bounds__(kProbeThreads)
void read_probe_kernel(const u32x4* __restrict__ base, int64_t n16, uint32_t* __restrict__ sums)
{
    __shared__ uint32_t part[kProbeThreads / 64];
    u32x4 acc = {0u, 0u, 0u, 0u};
    int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kProbeThreads;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = stream_load(base + i + k * stride);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc ^= v[k];
    }
    for (; i < n16; i += stride) acc ^= stream_load(base + i);
    uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) r ^= __shfl_xor(r, d, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int w = 0; w < kProbeThreads / 64; ++w) t ^= part[w];
        sums[blockIdx.x] = t;
    }
}

}  // namespace

hipError_t launch_read_probe(const void* buf, int64_t bytes, uint32_t* sums, hipStream_t stream)
{
    const LaunchEvents ev = take_launch_events();
    if (ev.start != nullptr || ev.stop != nullptr)
        hipExtLaunchKernelGGL(read_probe_kernel, dim3(kReadProbeBlocks), dim3(kProbeThreads), 0u, stream,
                              ev.start, ev.stop, 0u, static_cast<const u32x4*>(buf), bytes / 16, sums);
    else
        hipLaunchKernelGGL(read_probe_kernel, dim3(kReadProbeBlocks), dim3(kProbeThreads), 0, stream,
                           static_cast<const u32x4*>(buf), bytes / 16, sums);
    return hipGetLastError();
}

}  // namespace e3
