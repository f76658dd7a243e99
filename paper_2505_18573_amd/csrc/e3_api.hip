// C ABI of libe3: argument checks on the host, then kernel launches.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>

#include "../../include/e3.h"
#include "../../include/e3_measure.h"
#include "vocab_pass.h"

namespace {

int check_logits(const void* logits, int dtype, int64_t rows, int64_t V, int64_t row_stride)
{
    if (dtype != E3_F32 && dtype != E3_BF16) return E3_ERR_DTYPE;
    if (rows < 0 || V < 1 || row_stride < V) return E3_ERR_SHAPE;
    if (V > (int64_t)0x7FFFFFFF - 8192 || rows > (int64_t)0x7FFFFFFF) return E3_ERR_SHAPE;
    if (!e3::vocab_pass_fits(V)) return E3_ERR_SHAPE;      // beyond ~1M columns
    if (rows == 0) return E3_OK;
    if (logits == nullptr) return E3_ERR_NULL;
    const int64_t esz = dtype == E3_F32 ? 4 : 2;
    if ((reinterpret_cast<uintptr_t>(logits) & 15u) != 0 || ((row_stride * esz) & 15) != 0)
        return E3_ERR_ALIGN;
    return E3_OK;
}

int check_tau(const float* tau_rows, float tau_scalar)
{
    if (tau_rows != nullptr) return E3_OK;
    return (std::isfinite(tau_scalar) && tau_scalar > 0.0f) ? E3_OK : E3_ERR_VALUE;
}

// When a call's vocabulary pass is followed by a reduction kernel, the measurement hook's stop
// event goes to that last kernel: take it out of the pending pair and leave the start event
// for the vocabulary pass.
hipEvent_t split_stop_event()
{
    const e3::LaunchEvents ev = e3::take_launch_events();
    e3::set_launch_events(ev.start, nullptr);
    return ev.stop;
}

}  // namespace

extern "C" const char* e3_strerror(int status)
{
    switch (status) {
        case E3_OK: return "ok";
        case E3_ERR_NULL: return "a required pointer is NULL";
        case E3_ERR_SHAPE: return "bad shape (rows < 0, V < 1, row_stride < V, or too large)";
        case E3_ERR_DTYPE: return "unknown dtype";
        case E3_ERR_ALIGN: return "logits base or row pitch is not 16-byte aligned";
        case E3_ERR_VALUE: return "scalar argument outside its domain";
        case E3_ERR_WORKSPACE: return "batch exceeds what the library-owned scratch holds";
        case E3_ERR_LAUNCH: return "HIP launch failed";
        default: return "unknown status";
    }
}

extern "C" size_t e3_workspace_bytes(int64_t rows, int64_t V)
{
    return e3::vocab_pass_workspace_bytes(rows, V);
}

extern "C" int e3_sample_entropy(const void* logits, int dtype, int64_t rows, int64_t V,
                                 int64_t row_stride, const float* tau_rows, float tau_scalar,
                                 uint64_t seed, uint64_t row_base,
                                 int32_t* token_out, float* logp_out, float* entropy_out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream)
{
    int rc = check_logits(logits, dtype, rows, V, row_stride);
    if (rc != E3_OK) return rc;
    rc = check_tau(tau_rows, tau_scalar);
    if (rc != E3_OK) return rc;
    if (rows == 0) return E3_OK;
    if (token_out == nullptr) return E3_ERR_NULL;

    e3::VocabPassArgs a{};
    a.logits = logits; a.rows = rows; a.V = V; a.row_stride = row_stride;
    a.tau_rows = tau_rows; a.tau_scalar = tau_scalar;
    a.seed = seed; a.row_base = row_base;
    a.target_ids = nullptr;
    a.token_out = token_out; a.logp_out = logp_out; a.entropy_out = entropy_out;
    hipError_t err = e3::launch_vocab_pass(a, dtype == E3_BF16, true, workspace, workspace_bytes,
                                           static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E3_OK : E3_ERR_LAUNCH;
}

extern "C" int e3_sample_entropy_noalloc(const void* logits, int dtype, int64_t rows, int64_t V,
                                         int64_t row_stride, const float* tau_rows, float tau_scalar,
                                         uint64_t seed, uint64_t row_base,
                                         int32_t* token_out, float* logp_out, float* entropy_out,
                                         void* hip_stream)
{
    int rc = check_logits(logits, dtype, rows, V, row_stride);
    if (rc != E3_OK) return rc;
    rc = check_tau(tau_rows, tau_scalar);
    if (rc != E3_OK) return rc;
    if (rows > e3::static_scratch_max_rows()) return E3_ERR_WORKSPACE;
    if (rows == 0) return E3_OK;
    if (token_out == nullptr) return E3_ERR_NULL;
    void* ws = nullptr;
    size_t ws_bytes = 0;
    if (e3::static_scratch(&ws, &ws_bytes) != hipSuccess) return E3_ERR_LAUNCH;

    e3::VocabPassArgs a{};
    a.logits = logits; a.rows = rows; a.V = V; a.row_stride = row_stride;
    a.tau_rows = tau_rows; a.tau_scalar = tau_scalar;
    a.seed = seed; a.row_base = row_base;
    a.target_ids = nullptr;
    a.token_out = token_out; a.logp_out = logp_out; a.entropy_out = entropy_out;
    hipError_t err = e3::launch_vocab_pass(a, dtype == E3_BF16, true, ws, ws_bytes,
                                           static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E3_OK : E3_ERR_LAUNCH;
}

extern "C" int e3_time_next_launch(void* start_event, void* stop_event)
{
    e3::set_launch_events(static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event));
    return E3_OK;
}

extern "C" int e3_read_probe(const void* buf, int64_t bytes, uint32_t* sums_out, void* hip_stream)
{
    if (bytes < 0 || (bytes & 15) != 0) return E3_ERR_SHAPE;
    if (sums_out == nullptr || (buf == nullptr && bytes > 0)) return E3_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0) return E3_ERR_ALIGN;
    hipError_t err = e3::launch_read_probe(buf, bytes, sums_out, static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E3_OK : E3_ERR_LAUNCH;
}

extern "C" int e3_sample_restricted(const void* logits, int dtype, int64_t rows, int64_t V,
                                    int64_t row_stride, const float* tau_rows, float tau_scalar,
                                    int32_t top_k, float top_p, uint64_t seed, uint64_t row_base,
                                    int32_t* token_out, float* logp_out, int32_t* kept_out,
                                    void* hip_stream)
{
    int rc = check_logits(logits, dtype, rows, V, row_stride);
    if (rc != E3_OK) return rc;
    rc = check_tau(tau_rows, tau_scalar);
    if (rc != E3_OK) return rc;
    if (top_k < 0 || !(top_p > 0.0f) || !std::isfinite(top_p)) return E3_ERR_VALUE;
    // a small top_k is served by selection, for both logit types; everything else needs the
    // histogram of all bit patterns, which exists for 16-bit patterns only
    const bool by_selection = e3::sample_select_serves(top_k);
    if (!by_selection && dtype == E3_F32) return E3_ERR_VALUE;
    if (rows == 0) return E3_OK;
    if (token_out == nullptr) return E3_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t err = by_selection
        ? e3::launch_sample_select(logits, dtype == E3_BF16, rows, V, row_stride, tau_rows, tau_scalar,
                                   top_k, top_p, seed, row_base, token_out, logp_out, kept_out, stream)
        : e3::launch_sample_restricted(logits, rows, V, row_stride, tau_rows, tau_scalar, top_k, top_p,
                                       seed, row_base, token_out, logp_out, kept_out, stream);
    return err == hipSuccess ? E3_OK : E3_ERR_LAUNCH;
}

extern "C" int e3_logprob_entropy_gap(const void* logits, int dtype, int64_t rows, int64_t V,
                                      int64_t row_stride, const int32_t* target_ids,
                                      const uint8_t* row_mask, const float* tau_rows, float tau_scalar,
                                      float* logp_out, float* entropy_out, float* gap_out,
                                      double* entropy_sum_out, double* gap_sum_out,
                                      int64_t* count_out,
                                      void* workspace, size_t workspace_bytes, void* hip_stream)
{
    int rc = check_logits(logits, dtype, rows, V, row_stride);
    if (rc != E3_OK) return rc;
    rc = check_tau(tau_rows, tau_scalar);
    if (rc != E3_OK) return rc;
    if (rows > 0 && entropy_out == nullptr) return E3_ERR_NULL;
    if (logp_out != nullptr && target_ids == nullptr) return E3_ERR_NULL;
    if (gap_sum_out != nullptr && gap_out == nullptr) return E3_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool h_sum = entropy_sum_out != nullptr || count_out != nullptr, g_sum = gap_sum_out != nullptr;
    // measurement hook: the stop event belongs to the call's last kernel
    hipEvent_t stop_last = nullptr;
    if (rows > 0 && (h_sum || g_sum)) stop_last = split_stop_event();

    if (rows > 0) {
        e3::VocabPassArgs a{};
        a.logits = logits; a.rows = rows; a.V = V; a.row_stride = row_stride;
        a.tau_rows = tau_rows; a.tau_scalar = tau_scalar;
        a.target_ids = target_ids;
        a.token_out = nullptr; a.logp_out = logp_out; a.entropy_out = entropy_out;
        a.gap_out = gap_out;
        if (e3::launch_vocab_pass(a, dtype == E3_BF16, false, workspace, workspace_bytes, stream)
            != hipSuccess)
            return E3_ERR_LAUNCH;
    }
    // also for rows == 0: sums and count are then written as 0
    if (h_sum) {
        if (e3::launch_entropy_reduce(entropy_out, row_mask, rows, entropy_sum_out, count_out,
                                      stream, g_sum ? nullptr : stop_last) != hipSuccess)
            return E3_ERR_LAUNCH;
    }
    if (g_sum) {
        if (e3::launch_entropy_reduce(gap_out, row_mask, rows, gap_sum_out, nullptr, stream, stop_last)
            != hipSuccess)
            return E3_ERR_LAUNCH;
    }
    return E3_OK;
}

extern "C" int e3_logprob_entropy_advantages(const void* logits, int dtype, int64_t rows, int64_t V,
                                            int64_t row_stride, const int32_t* target_ids,
                                            const uint8_t* row_mask, const float* tau_rows,
                                            float tau_scalar, float* logp_out, float* entropy_out,
                                            double* entropy_sum_out, int64_t* entropy_count_out,
                                            const float* rewards, const int32_t* group_offsets,
                                            int32_t num_groups, int32_t ddof, float eps, float* adv_out,
                                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    int rc = check_logits(logits, dtype, rows, V, row_stride);
    if (rc != E3_OK) return rc;
    rc = check_tau(tau_rows, tau_scalar);
    if (rc != E3_OK) return rc;
    if (rows > 0 && entropy_out == nullptr) return E3_ERR_NULL;
    if (logp_out != nullptr && target_ids == nullptr) return E3_ERR_NULL;
    if (num_groups < 0) return E3_ERR_SHAPE;
    if (ddof != 0 && ddof != 1) return E3_ERR_VALUE;
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return E3_ERR_VALUE;
    if (num_groups > 0 && (rewards == nullptr || group_offsets == nullptr || adv_out == nullptr))
        return E3_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    e3::VocabPassArgs a{};
    a.logits = logits; a.rows = rows; a.V = V; a.row_stride = row_stride;
    a.tau_rows = tau_rows; a.tau_scalar = tau_scalar;
    a.target_ids = target_ids;
    a.token_out = nullptr; a.logp_out = logp_out; a.entropy_out = entropy_out;
    a.adv_rewards = rewards; a.adv_offsets = group_offsets; a.adv_groups = num_groups;
    a.adv_ddof = ddof; a.adv_eps = eps; a.adv_out = adv_out;
    const bool h_sum = entropy_sum_out != nullptr || entropy_count_out != nullptr;
    hipEvent_t stop_last = nullptr;
    if (rows > 0 && h_sum) stop_last = split_stop_event();      // measurement hook, see above
    if (e3::launch_vocab_pass(a, dtype == E3_BF16, false, workspace, workspace_bytes, stream) != hipSuccess)
        return E3_ERR_LAUNCH;
    if (h_sum) {
        if (e3::launch_entropy_reduce(entropy_out, row_mask, rows, entropy_sum_out, entropy_count_out,
                                      stream, stop_last) != hipSuccess)
            return E3_ERR_LAUNCH;
    }
    return E3_OK;
}

extern "C" int e3_logprob_entropy(const void* logits, int dtype, int64_t rows, int64_t V,
                                  int64_t row_stride, const int32_t* target_ids,
                                  const uint8_t* row_mask, const float* tau_rows, float tau_scalar,
                                  float* logp_out, float* entropy_out,
                                  double* entropy_sum_out, int64_t* entropy_count_out,
                                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return e3_logprob_entropy_gap(logits, dtype, rows, V, row_stride, target_ids, row_mask, tau_rows,
                                  tau_scalar, logp_out, entropy_out, nullptr, entropy_sum_out, nullptr,
                                  entropy_count_out, workspace, workspace_bytes, hip_stream);
}

extern "C" int e3_grpo_advantages(const float* rewards, const int32_t* group_offsets,
                                  int32_t num_groups, int32_t ddof, float eps,
                                  float* adv_out, void* hip_stream)
{
    if (num_groups < 0) return E3_ERR_SHAPE;
    if (ddof != 0 && ddof != 1) return E3_ERR_VALUE;
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return E3_ERR_VALUE;
    if (num_groups == 0) return E3_OK;
    if (rewards == nullptr || group_offsets == nullptr || adv_out == nullptr) return E3_ERR_NULL;
    hipError_t err = e3::launch_grpo_advantages(rewards, group_offsets, num_groups, ddof, eps,
                                                adv_out, static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E3_OK : E3_ERR_LAUNCH;
}

extern "C" int e3_grpo_objective(const float* logp_new, const float* logp_old,
                                 const int32_t* seq_offsets, const float* adv, int32_t num_seqs,
                                 const int32_t* group_offsets, int32_t num_groups, float clip_eps,
                                 float* token_term_out, double* seq_mean_out, double* objective_out,
                                 void* hip_stream)
{
    if (num_seqs < 0 || num_groups < 0) return E3_ERR_SHAPE;
    if (!(clip_eps >= 0.0f) || !std::isfinite(clip_eps)) return E3_ERR_VALUE;
    if (objective_out == nullptr || group_offsets == nullptr) return E3_ERR_NULL;
    if (num_seqs > 0 && (logp_new == nullptr || logp_old == nullptr || seq_offsets == nullptr ||
                         adv == nullptr || seq_mean_out == nullptr))
        return E3_ERR_NULL;
    hipError_t err = e3::launch_grpo_objective(logp_new, logp_old, seq_offsets, adv, num_seqs,
                                               group_offsets, num_groups, clip_eps, token_term_out,
                                               seq_mean_out, objective_out,
                                               static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E3_OK : E3_ERR_LAUNCH;
}
