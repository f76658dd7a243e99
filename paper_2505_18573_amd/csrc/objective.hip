// Forward value of the GRPO clipped objective (Eq. 1 of arXiv 2505.18573, without the
// KL term the paper drops): per token min(r A, clip(r, 1-eps, 1+eps) A) with
// r = exp(logp_new - logp_old), averaged over the tokens of a rollout, then over the
// rollouts of a question, then over questions.  It consumes what the vocabulary pass
// (log-probs) and the advantage kernel (A) produce.  Two launches: one wave per rollout
// (fp64 sums, DPP reduction), then one workgroup that folds rollouts into questions and
// questions into the scalar in a fixed order (bit-reproducible).
#include "vocab_common.h"
#include "vocab_pass.h"

namespace e3 {

constexpr int kSeqsPerBlock = 4;

__global__ __launch_bounds__(kSeqsPerBlock * 64)
void grpo_seq_terms_kernel(const float* __restrict__ logp_new, const float* __restrict__ logp_old,
                           const int32_t* __restrict__ seq_offsets, const float* __restrict__ adv,
                           int32_t num_seqs, float clip_eps, float* __restrict__ token_term_out,
                           double* __restrict__ seq_mean_out)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * kSeqsPerBlock + (threadIdx.x >> 6);
    if (i >= num_seqs) return;
    const int64_t t0 = seq_offsets[i], t1 = seq_offsets[i + 1];
    const float A = adv[i];
    const float lo = 1.0f - clip_eps, hi = 1.0f + clip_eps;
    double acc = 0.0;
    for (int64_t t = t0 + lane; t < t1; t += 64) {
        const float r = __builtin_amdgcn_exp2f((logp_new[t] - logp_old[t]) * kLog2eF);
        const float rc = fminf(fmaxf(r, lo), hi);
        const float term = fminf(r * A, rc * A);
        if (token_term_out) token_term_out[t] = term;
        acc += (double)term;
    }
    acc = wave_sum(acc);
    if (lane == 0) seq_mean_out[i] = t1 > t0 ? acc / (double)(t1 - t0) : 0.0;
}

__global__ __launch_bounds__(1024)
void grpo_objective_reduce_kernel(const double* __restrict__ seq_mean,
                                  const int32_t* __restrict__ group_offsets, int32_t num_groups,
                                  double* objective_out)
{
    __shared__ double partial[16];
    double acc = 0.0;
    for (int32_t q = threadIdx.x; q < num_groups; q += 1024) {
        const int32_t i0 = group_offsets[q], i1 = group_offsets[q + 1];
        double g = 0.0;
        for (int32_t i = i0; i < i1; ++i) g += seq_mean[i];
        if (i1 > i0) acc += g / (double)(i1 - i0);
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) partial[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
        for (int w = 0; w < 16; ++w) total += partial[w];
        *objective_out = num_groups > 0 ? total / (double)num_groups : 0.0;
    }
}

hipError_t launch_grpo_objective(const float* logp_new, const float* logp_old,
                                 const int32_t* seq_offsets, const float* adv, int32_t num_seqs,
                                 const int32_t* group_offsets, int32_t num_groups, float clip_eps,
                                 float* token_term_out, double* seq_mean_out, double* objective_out,
                                 hipStream_t stream)
{
    if (num_seqs > 0) {
        const unsigned blocks = (unsigned)((num_seqs + kSeqsPerBlock - 1) / kSeqsPerBlock);
        hipLaunchKernelGGL(grpo_seq_terms_kernel, dim3(blocks), dim3(kSeqsPerBlock * 64), 0, stream,
                           logp_new, logp_old, seq_offsets, adv, num_seqs, clip_eps, token_term_out,
                           seq_mean_out);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    hipLaunchKernelGGL(grpo_objective_reduce_kernel, dim3(1), dim3(1024), 0, stream,
                       seq_mean_out, group_offsets, num_groups, objective_out);
    return hipGetLastError();
}

}  // namespace e3
