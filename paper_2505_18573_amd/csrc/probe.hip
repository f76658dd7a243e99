// Read-bandwidth probe for gfx950: streams a device buffer once with the access pattern
// of the vocabulary pass (16-byte non-temporal loads, a wave instruction covering 1 KiB
// of contiguous memory, a whole 16-KiB run per wave in flight and refilled as it is
// consumed, workgroups of eight waves owning contiguous stretches) and does nothing else
// but fold the data into per-workgroup xor checksums.  It contains no arithmetic of the
// method; the benchmark times it on its own logit buffers so that the kernels' achieved
// GB/s can be read against what a pure read of the same bytes reaches on the same machine.
// (Measured on MI355X against flat grid-stride reads of 1024 to 8192 workgroups and
// against shallower prefetch: this shape was the fastest or within 2 % of it from 156 MB
// to 10 GB.)
#include "vocab_common.h"
#include "vocab_pass.h"
#include <hip/hip_ext.h>

namespace e3 {
namespace {

constexpr int kProbeWaves = 8;
constexpr int kRunVecs = 1024;            // 16-byte vectors per run: 16 sweeps x 64 lanes

__global__ __launch_bounds__(kProbeWaves * 64)
void read_probe_kernel(const u32x4* __restrict__ base, int64_t n16, int64_t runs_per_block,
                       uint32_t* __restrict__ sums)
{
    __shared__ uint32_t part[kProbeWaves];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t runs = n16 / kRunVecs;
    const int64_t first = (int64_t)blockIdx.x * runs_per_block;
    const int64_t last = first + runs_per_block < runs ? first + runs_per_block : runs;
    u32x4 acc = {0u, 0u, 0u, 0u};
    u32x4 buf[16];
    int64_t run = first + wave;
    if (run < last) {
#pragma unroll
        for (int i = 0; i < 16; ++i) buf[i] = stream_load(base + run * kRunVecs + i * 64 + lane);
    }
    for (; run < last; run += kProbeWaves) {
        const bool more = run + kProbeWaves < last;
        const u32x4* next = base + (run + kProbeWaves) * kRunVecs + lane;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            acc ^= buf[i];
            if (more) buf[i] = stream_load(next + i * 64);
        }
    }
    // what does not fill a run: the last workgroup reads it flat
    if (blockIdx.x == gridDim.x - 1)
        for (int64_t v = runs * kRunVecs + threadIdx.x; v < n16; v += kProbeWaves * 64) acc ^= base[v];
    uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) r ^= __shfl_xor(r, d, 64);
    if (lane == 0) part[wave] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int w = 0; w < kProbeWaves; ++w) t ^= part[w];
        sums[blockIdx.x] = t;
    }
}

__global__ void zero_sums_kernel(uint32_t* sums, int from)
{
    const int i = from + blockIdx.x * blockDim.x + threadIdx.x;
    if (i < kReadProbeBlocks) sums[i] = 0u;
}

}  // namespace

hipError_t launch_read_probe(const void* buf, int64_t bytes, uint32_t* sums, hipStream_t stream)
{
    // 38 runs of 16 KiB per workgroup (two bf16 rows of 151,936 columns), but never
    // more workgroups than checksum slots
    const int64_t n16 = bytes / 16;
    const int64_t runs = n16 / kRunVecs;
    int64_t per_block = 38;
    if ((runs + per_block - 1) / per_block > kReadProbeBlocks)
        per_block = (runs + kReadProbeBlocks - 1) / kReadProbeBlocks;
    int64_t blocks = (runs + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (blocks < kReadProbeBlocks) {
        hipLaunchKernelGGL(zero_sums_kernel, dim3((kReadProbeBlocks + 255) / 256), dim3(256), 0, stream,
                           sums, (int)blocks);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    const LaunchEvents ev = take_launch_events();
    if (ev.start != nullptr || ev.stop != nullptr)
        hipExtLaunchKernelGGL(read_probe_kernel, dim3((unsigned)blocks), dim3(kProbeWaves * 64), 0u, stream,
                              ev.start, ev.stop, 0u, static_cast<const u32x4*>(buf), n16, per_block, sums);
    else
        hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)blocks), dim3(kProbeWaves * 64), 0, stream,
                           static_cast<const u32x4*>(buf), n16, per_block, sums);
    return hipGetLastError();
}

}  // namespace e3
