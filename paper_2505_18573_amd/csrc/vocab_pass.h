// Internal launch interface between the C ABI (e3_api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace e3 {

struct VocabPassArgs {
    const void* logits;
    int64_t rows, V, row_stride;      // row_stride in elements
    const float* tau_rows;            // device [rows] or nullptr
    float tau_scalar;
    uint64_t seed, row_base;          // sampling only
    const int32_t* target_ids;        // training side, device [rows] or nullptr
    int32_t* token_out;               // sampling only
    float* logp_out;                  // nullable
    float* entropy_out;               // nullable
    float* gap_out;                   // nullable: measured logit gap (Appendix A's Delta)
    // training side, optional: rollout groups whose advantages (Eq. 2) are computed in the
    // same launch (adv_groups == 0: none)
    const float* adv_rewards;
    const int32_t* adv_offsets;
    int32_t adv_groups, adv_ddof;
    float adv_eps;
    float* adv_out;
};

// `workspace` (device, 16-byte aligned, nullable) lets small batches be cut across
// many workgroups; without it, or when it is too small, whole rows stay in one workgroup.
hipError_t launch_vocab_pass(const VocabPassArgs& a, bool is_bf16, bool sample,
                             void* workspace, size_t workspace_bytes, hipStream_t stream);

// events (nullable) that the next launch_vocab_pass of this host thread attaches to its
// kernel dispatch(es); consumed by that launch
void set_launch_events(hipEvent_t start, hipEvent_t stop);
struct LaunchEvents {
    hipEvent_t start, stop;
};
LaunchEvents take_launch_events();

// upper bound of the workspace the small-batch path can use for this shape (0: none)
size_t vocab_pass_workspace_bytes(int64_t rows, int64_t V);

// Library-owned scratch (a file-scope device array) that stands in for the caller workspace:
// address of the current device's copy and its size; rows beyond static_scratch_max_rows()
// are not served from it.  Looks the address up on the first call on a device.
hipError_t static_scratch(void** ptr_out, size_t* bytes_out);
int64_t static_scratch_max_rows();

// false when V is so large that the per-workgroup tables do not fit LDS
bool vocab_pass_fits(int64_t V);

// stop_event (nullable): attached to this dispatch, holds the time the kernel ended
hipError_t launch_entropy_reduce(const float* entropy, const uint8_t* mask, int64_t rows,
                                 double* sum_out, int64_t* count_out, hipStream_t stream,
                                 hipEvent_t stop_event = nullptr);

// top-k / top-p restricted sampling of bf16 rows (one workgroup per row)
hipError_t launch_sample_restricted(const void* logits, int64_t rows, int64_t V, int64_t row_stride,
                                    const float* tau_rows, float tau_scalar, int32_t top_k, float top_p,
                                    uint64_t seed, uint64_t row_base, int32_t* token_out,
                                    float* logp_out, int32_t* kept_out, hipStream_t stream);

// top-k (<= 256, see sample_select_serves) / top-p restricted sampling by selection, bf16 and
// fp32 rows (one workgroup per row)
bool sample_select_serves(int32_t top_k);
hipError_t launch_sample_select(const void* logits, bool is_bf16, int64_t rows, int64_t V, int64_t row_stride,
                                const float* tau_rows, float tau_scalar, int32_t top_k, float top_p,
                                uint64_t seed, uint64_t row_base, int32_t* token_out,
                                float* logp_out, int32_t* kept_out, hipStream_t stream);

// read-bandwidth probe: kReadProbeBlocks xor checksums of `bytes` (multiple of 16) bytes
constexpr int kReadProbeBlocks = 2048;
hipError_t launch_read_probe(const void* buf, int64_t bytes, uint32_t* sums, hipStream_t stream);

hipError_t launch_grpo_advantages(const float* rewards, const int32_t* offsets, int32_t num_groups,
                                  int32_t ddof, float eps, float* adv_out, hipStream_t stream);

hipError_t launch_grpo_objective(const float* logp_new, const float* logp_old,
                                 const int32_t* seq_offsets, const float* adv, int32_t num_seqs,
                                 const int32_t* group_offsets, int32_t num_groups, float clip_eps,
                                 float* token_term_out, double* seq_mean_out, double* objective_out,
                                 hipStream_t stream);

}  // namespace e3
