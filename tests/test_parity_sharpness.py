"""Would the comparisons of the library with the oracle notice a mistake?

Each case runs an existing library-vs-oracle test with ONE mistake planted in the oracle
(on the CPU; see the `wrong_oracle` fixture) and expects it to fail.  The tests named here
pass against the real oracle in the ordinary run.
"""
import importlib

import pytest

HOST_CASES = [
    # host-side library code (no GPU): ranks, Algorithm 1, bounds, the gap form of the update
    ("tests.test_budgets", "test_ranks_match_oracle_bit_exact",
     "k_out[i] = (double)(ahead + 1) / (double)n;", "k_out[i] = (double)ahead / (double)n;"),
    ("tests.test_budgets", "test_budgets_match_oracle_bit_exact",
     "(int64_t)floor((double)rem * k[i] / sum_k);", "(int64_t)floor((double)rem * k[i] / sum_k + 0.5);"),
    ("tests.test_budgets", "test_bounds_match_oracle",
     "int64_t hi = (int64_t)G + (int64_t)step * passes_done;", "int64_t hi = (int64_t)G + (int64_t)step * passes_done + 1;"),
    ("tests.test_gap", "test_update_gap_matches_oracle_on_host",
     "double next = tau_t * (1.0 + tau_t * log(target / H_t) / delta);",
     "double next = tau_t * (1.0 + tau_t * log(target / H_t) / delta * 1.0001);"),
]

GPU_CASES = [
    ("tests.test_restricted", "test_decode_rows_full_vocab",       # distinct top values: C_j = k is hit exactly
     "while (LV_END(jk) < (int64_t)top_k) ++jk;", "while (LV_END(jk) <= (int64_t)top_k) ++jk;"),
    ("tests.test_restricted", "test_top_k_exactly_on_a_level_boundary",
     "while (LV_END(jk) < (int64_t)top_k) ++jk;", "while (LV_END(jk) < (int64_t)top_k - 1) ++jk;"),
    ("tests.test_restricted", "test_repeated_values_and_signed_zeros",
     "M += (double)(e - i) * exp((z - z1) / tau);", "M += exp((z - z1) / tau);"),
    ("tests.test_restricted", "test_cuts_among_negative_values_and_back",
     "/ tau - log(lv_M[jp]);", "/ tau - log(lv_M[jp]) * 1.0003;"),
    ("tests.test_restricted", "test_shapes_and_tails",
     "e3o_noise_word(seed, grow, 3u, it[lv_first[j]].bits)", "e3o_noise_word(seed, grow, 3u, (uint32_t)j)"),
    ("tests.test_gap", "test_gap_parity_on_gpu", "weighted += gap * e;", "weighted += gap * e * 1.0003;"),
    ("tests.test_objective", "test_objective_parity_on_gpu", "double term = a < b ? a : b;", "double term = a > b ? a : b;"),
    ("tests.test_gpu_parity", "test_advantages_group_shapes",
     "double sigma = sqrt(ss / (double)(n - ddof));", "double sigma = sqrt(ss / (double)(n - ddof)) * 1.00001;"),
    ("tests.test_budgets", "test_budgets_feed_advantages_on_gpu",
     "adv_out[i] = ((double)rewards[i] - mean) / (sigma + eps);", "adv_out[i] = ((double)rewards[i] - mean * 1.0001) / (sigma + eps);"),
]


def _expect_failure(module, func, find, replace, plant):
    fn = getattr(importlib.import_module(module), func)
    kwargs = {"test_shapes_and_tails": {"V": 1000}, "test_decode_rows_full_vocab": {"k": 50, "p": 1.0}}.get(func, {})
    plant(find, replace)
    with pytest.raises(AssertionError):
        fn(**kwargs)


@pytest.mark.parametrize("module,func,find,replace", HOST_CASES, ids=[c[1] for c in HOST_CASES])
def test_host_comparisons_notice_a_wrong_oracle(module, func, find, replace, wrong_oracle):
    _expect_failure(module, func, find, replace, wrong_oracle)


@pytest.mark.gpu
@pytest.mark.parametrize("module,func,find,replace", GPU_CASES, ids=[c[1] for c in GPU_CASES])
def test_gpu_comparisons_notice_a_wrong_oracle(module, func, find, replace, wrong_oracle):
    _expect_failure(module, func, find, replace, wrong_oracle)
