"""MI355X-native hot path of E3 (arXiv 2505.18573): fused temperature-softmax entropy,
token log-prob and Gumbel-max sampling over [rows, V] logits, GRPO group advantages over
CSR groups, and the closed-form temperature scheduler.  The arithmetic lives in libe3.so
(HIP, gfx950); this package is its ctypes binding plus seeded workload generators."""
from .binding import (E3_BF16, E3_F32, E3Error, e3_allocate_budgets, e3_budget_bounds,
                      e3_difficulty_ranks, e3_grpo_advantages, e3_grpo_objective, e3_logprob_entropy_gap, e3_read_probe, e3_time_next_launch,
                      e3_temperature_update_gap, e3_logprob_entropy, e3_logprob_entropy_advantages,
                      e3_sample_entropy, e3_sample_entropy_noalloc, e3_sample_restricted, e3_strerror, e3_temperature_update,
                      e3_workspace_bytes, lib, new_workspace)

__all__ = ["E3_BF16", "E3_F32", "E3Error", "e3_allocate_budgets", "e3_budget_bounds",
           "e3_difficulty_ranks", "e3_grpo_advantages", "e3_grpo_objective", "e3_logprob_entropy_gap", "e3_read_probe", "e3_time_next_launch",
           "e3_temperature_update_gap", "e3_logprob_entropy", "e3_logprob_entropy_advantages",
           "e3_sample_entropy", "e3_sample_entropy_noalloc", "e3_sample_restricted", "e3_strerror", "e3_temperature_update", "e3_workspace_bytes",
           "lib", "new_workspace"]
