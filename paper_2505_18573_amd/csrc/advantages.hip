// Group-relative advantage (Eq. 2 of arXiv 2505.18573) over CSR-stored rollout
// groups: A_i = (r_i - mean(r)) / std(r).  One wave per group, two passes over the
// group's rewards (mean, then squared deviations), sums in fp64.  Groups whose
// rewards are all identical get exactly 0 (Section 4.2), decided by max == min.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vocab_pass.h"

namespace e3 {

constexpr int kGroupsPerBlock = 4;

__global__ __launch_bounds__(kGroupsPerBlock * 64)
void grpo_advantages_kernel(const float* __restrict__ rewards, const int32_t* __restrict__ offsets,
                            int32_t num_groups, int32_t ddof, float eps, float* __restrict__ adv)
{
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * kGroupsPerBlock + (threadIdx.x >> 6);
    if (g >= num_groups) return;
    const int64_t lo = offsets[g], hi = offsets[g + 1];
    const int64_t n = hi - lo;
    if (n <= 0) return;

    double sum = 0.0;
    float rmax = -INFINITY, rmin = INFINITY;
    for (int64_t i = lo + lane; i < hi; i += 64) {
        const float r = rewards[i];
        sum += (double)r;
        rmax = fmaxf(rmax, r);
        rmin = fminf(rmin, r);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        sum += __shfl_xor(sum, off, 64);
        rmax = fmaxf(rmax, __shfl_xor(rmax, off, 64));
        rmin = fminf(rmin, __shfl_xor(rmin, off, 64));
    }
    if (rmax == rmin) {
        for (int64_t i = lo + lane; i < hi; i += 64) adv[i] = 0.0f;
        return;
    }
    const double mean = sum / (double)n;
    double ss = 0.0;
    for (int64_t i = lo + lane; i < hi; i += 64) {
        const double d = (double)rewards[i] - mean;
        ss += d * d;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    const double denom = sqrt(ss / (double)(n - ddof)) + (double)eps;
    for (int64_t i = lo + lane; i < hi; i += 64)
        adv[i] = (float)(((double)rewards[i] - mean) / denom);
}

hipError_t launch_grpo_advantages(const float* rewards, const int32_t* offsets, int32_t num_groups,
                                  int32_t ddof, float eps, float* adv_out, hipStream_t stream)
{
    if (num_groups == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((num_groups + kGroupsPerBlock - 1) / kGroupsPerBlock);
    hipLaunchKernelGGL(grpo_advantages_kernel, dim3(blocks), dim3(kGroupsPerBlock * 64), 0, stream,
                       rewards, offsets, num_groups, ddof, eps, adv_out);
    return hipGetLastError();
}

}  // namespace e3
