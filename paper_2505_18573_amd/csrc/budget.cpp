// Dynamic rollout budgets of arXiv 2505.18573 (Section 4.1): difficulty ranking of
// the questions, Algorithm 1 (per-question rollout counts with a constant batch total)
// and the G_min / G_max curriculum.  Host-side integer code; the counts it returns
// become the CSR group offsets that e3_grpo_advantages consumes.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <vector>

#include "../../include/e3.h"

extern "C" int e3_difficulty_ranks(const double* cum_reward, const int64_t* cum_rollouts,
                                   int64_t num_questions, double* k_out)
{
    if (num_questions < 0) return E3_ERR_SHAPE;
    if (num_questions == 0) return E3_OK;
    if (cum_reward == nullptr || cum_rollouts == nullptr || k_out == nullptr) return E3_ERR_NULL;
    const size_t n = static_cast<size_t>(num_questions);
    std::vector<double> avg(n);
    for (size_t i = 0; i < n; ++i) {
        if (cum_rollouts[i] < 0) return E3_ERR_VALUE;
        avg[i] = cum_rollouts[i] > 0 ? cum_reward[i] / static_cast<double>(cum_rollouts[i]) : 0.0;
        if (std::isnan(avg[i])) return E3_ERR_VALUE;
    }
    // rank 1 = highest average reward; a stable sort keeps index order among equals
    std::vector<int64_t> by_reward(n);
    std::iota(by_reward.begin(), by_reward.end(), int64_t{0});
    std::stable_sort(by_reward.begin(), by_reward.end(),
                     [&](int64_t a, int64_t b) { return avg[a] > avg[b]; });
    for (size_t pos = 0; pos < n; ++pos)
        k_out[by_reward[pos]] = static_cast<double>(pos + 1) / static_cast<double>(n);
    return E3_OK;
}

extern "C" int e3_allocate_budgets(const double* k, int32_t B, int32_t G, int32_t G_min,
                                   int32_t G_max, int32_t* G_out, int32_t* offsets_out)
{
    if (B < 0) return E3_ERR_SHAPE;
    if (G_min < 0 || G_min > G || G > G_max) return E3_ERR_VALUE;
    if (static_cast<int64_t>(B) * G_max > INT32_MAX) return E3_ERR_SHAPE;   // offsets are int32
    if (B == 0) {
        if (offsets_out != nullptr) offsets_out[0] = 0;
        return E3_OK;
    }
    if (k == nullptr || G_out == nullptr) return E3_ERR_NULL;
    double k_sum = 0.0;
    for (int32_t i = 0; i < B; ++i) {
        if (!std::isfinite(k[i]) || k[i] < 0.0) return E3_ERR_VALUE;
        k_sum += k[i];
    }
    if (!(k_sum > 0.0)) return E3_ERR_VALUE;

    const int64_t budget = static_cast<int64_t>(B) * G;
    const int64_t spare = budget - static_cast<int64_t>(B) * G_min;
    std::vector<int32_t> g(static_cast<size_t>(B));
    int64_t spent = 0;
    for (int32_t i = 0; i < B; ++i) {
        const double share = std::floor(static_cast<double>(spare) * k[i] / k_sum);
        const int64_t want = static_cast<int64_t>(G_min) + static_cast<int64_t>(share);
        g[i] = static_cast<int32_t>(std::min<int64_t>(want, G_max));
        spent += g[i];
    }
    // leftovers: one rollout per question per pass, hardest first, never above G_max
    std::vector<int32_t> hardest_first(static_cast<size_t>(B));
    std::iota(hardest_first.begin(), hardest_first.end(), 0);
    std::stable_sort(hardest_first.begin(), hardest_first.end(),
                     [&](int32_t a, int32_t b) { return k[a] > k[b]; });
    int64_t left = budget - spent;
    while (left > 0) {
        bool moved = false;
        for (int32_t q : hardest_first) {
            if (left == 0) break;
            if (g[q] < G_max) { ++g[q]; --left; moved = true; }
        }
        if (!moved) return E3_ERR_VALUE;       // unreachable while G <= G_max
    }
    std::copy(g.begin(), g.end(), G_out);
    if (offsets_out != nullptr) {
        offsets_out[0] = 0;
        for (int32_t i = 0; i < B; ++i) offsets_out[i + 1] = offsets_out[i] + g[i];
    }
    return E3_OK;
}

extern "C" int e3_budget_bounds(int32_t G, int32_t passes_done, int32_t step, int32_t G_min_limit,
                                int32_t G_max_limit, int32_t* G_min_out, int32_t* G_max_out)
{
    if (G_min_out == nullptr || G_max_out == nullptr) return E3_ERR_NULL;
    if (G < 0 || passes_done < 0 || step < 0 || G_min_limit < 0 || G_min_limit > G || G_max_limit < G)
        return E3_ERR_VALUE;
    const int64_t widen = static_cast<int64_t>(step) * passes_done;
    *G_min_out = static_cast<int32_t>(std::max<int64_t>(G_min_limit, G - widen));
    *G_max_out = static_cast<int32_t>(std::min<int64_t>(G_max_limit, G + widen));
    return E3_OK;
}
