// Group-relative advantage (Eq. 2 of arXiv 2505.18573) over CSR-stored rollout groups,
// stand-alone launch: one wave per group (advantages.h).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "advantages.h"
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
    advantages_of_group(rewards, offsets, g, ddof, eps, adv, lane);
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
