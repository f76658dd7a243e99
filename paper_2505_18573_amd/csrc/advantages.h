// Group-relative advantage (Eq. 2 of arXiv 2505.18573) of ONE rollout group, computed by
// one wave: A_i = (r_i - mean(r)) / std(r), two passes over the group's rewards (mean,
// then squared deviations), sums in fp64.  A group whose rewards are all identical gets
// exactly 0 (Section 4.2), decided by max == min.  Shared by the stand-alone kernel and by
// the training-side vocabulary pass, which can carry the groups along in the same launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace e3 {

__device__ __forceinline__ void advantages_of_group(const float* __restrict__ rewards,
                                                    const int32_t* __restrict__ offsets, int g,
                                                    int32_t ddof, float eps, float* __restrict__ adv,
                                                    int lane)
{
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

}  // namespace e3
