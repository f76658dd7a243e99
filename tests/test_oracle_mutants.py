"""Do the oracle's pins notice a mistake?  (not gpu)

Each case below plants ONE plausible mistake in a copy of the oracle's C source (a dropped
term, a wrong sign, a swapped operand, an off-by-one, a wrong index), compiles the copy on the
CPU, puts it behind the oracle's Python front end and runs the pins of the affected part.  At
least one pin must fail.  The unmodified source, built and swapped in the same way, must pass
every pin used here, so a failure is the mistake's doing and not the swap's.

Nothing here touches the GPU or the HIP library.
"""
import ctypes
import importlib
import os
import subprocess

import pytest

from oracle import e3_oracle as o

SRC = os.path.join(os.path.dirname(os.path.abspath(o.__file__)), "e3_oracle.c")

ENT = "tests.test_oracle_entropy"
SMP = "tests.test_oracle_sampling"
RNG = "tests.test_oracle_rng"
ADV = "tests.test_oracle_advantages"
TMP = "tests.test_oracle_temperature"
BUD = "tests.test_oracle_budgets"
GAP = "tests.test_oracle_gap"
OBJ = "tests.test_oracle_objective"
RES = "tests.test_oracle_restricted"

# pins of each part: (module, function, kwargs)
PINS = {
    "entropy": [(ENT, "test_uniform_logits_give_ln_V_for_any_tau", {}), (ENT, "test_worked_distributions", {}),
                (ENT, "test_limits_in_tau", {}), (ENT, "test_shift_and_scale_invariances", {}),
                (ENT, "test_decomposition_equals_textbook_definition", {}),
                (ENT, "test_delta_model_exact_form", {}), (ENT, "test_logprob_pins", {}),
                (ENT, "test_bf16_rows_are_widened_exactly", {}), (ENT, "test_per_row_tau_and_stride", {}),
                (ENT, "test_batch_mean_entropy_and_mask", {})],
    "rng": [(RNG, "test_published_known_answers", {}), (RNG, "test_second_implementation_agrees_word_for_word", {}),
            (RNG, "test_noise_addressing", {}), (RNG, "test_uniform_is_strictly_inside_unit_interval_and_fp32_exact", {}),
            (RNG, "test_gumbel_range_and_definition", {})],
    "sampling": [(SMP, "test_matches_restatement_on_tiny_rows", {"partition": (2, 3, 2)}),
                 (SMP, "test_matches_restatement_on_tiny_rows", {"partition": (8, 64, 16)}),
                 (SMP, "test_library_partition_shape", {}),
                 (SMP, "test_frequencies_follow_softmax_flat_and_tiled", {}),
                 (SMP, "test_determinism_and_row_base", {}),
                 (SMP, "test_exact_ties_go_to_the_lowest_index_and_are_flagged", {"level": 1}),
                 (SMP, "test_exact_ties_go_to_the_lowest_index_and_are_flagged", {"level": 2}),
                 (SMP, "test_equal_masses_and_single_column_rows", {}),
                 (SMP, "test_near_tie_flag_rule", {})],
    "advantages": [(ADV, "test_worked_group_1000", {}), (ADV, "test_binary_reward_closed_form", {}),
                   (ADV, "test_identical_rewards_give_zero", {}), (ADV, "test_moments_and_affine_invariance", {}),
                   (ADV, "test_csr_edges", {})],
    "temperature": [(TMP, "test_denominator_value", {}), (TMP, "test_fixed_point_alpha_one", {}),
                    (TMP, "test_eq4_values", {}), (TMP, "test_eq5_schedule", {}), (TMP, "test_guards_and_clamps", {})],
    "budgets": [(BUD, "test_ranks_hand_worked", {}), (BUD, "test_ranks_are_a_permutation_over_D", {}),
                (BUD, "test_algorithm1_hand_worked", {}), (BUD, "test_algorithm1_invariants_and_restatement", {}),
                (BUD, "test_bounds_curriculum", {})],
    "gap": [(GAP, "test_two_level_model_returns_delta_for_any_tau", {}), (GAP, "test_small_worked_rows", {}),
            (GAP, "test_invariances", {}), (GAP, "test_ties_entropy_through_the_decomposition", {}),
            (GAP, "test_gap_update_values_and_relation_to_eq4", {})],
    "objective": [(OBJ, "test_clip_cases_single_token", {}), (OBJ, "test_hand_worked_batch", {}),
                  (OBJ, "test_on_policy_value_is_mean_advantage", {}),
                  (OBJ, "test_matches_numpy_restatement_and_edge_cases", {})],
    "restricted": [(RES, "test_no_truncation_reproduces_the_softmax", {}),
                   (RES, "test_top_k_matches_numpy_partition_and_keeps_ties", {}),
                   (RES, "test_top_k_one_is_the_argmax_with_logp_zero", {}),
                   (RES, "test_top_p_matches_sort_and_cumsum_on_distinct_values", {}),
                   (RES, "test_hand_worked_dyadic_row", {}),
                   (RES, "test_draw_follows_the_truncated_softmax_with_repeated_values", {}),
                   (RES, "test_draw_matches_a_numpy_restatement", {"top_k": 12, "top_p": 0.9}),
                   (RES, "test_draw_matches_a_numpy_restatement", {"top_k": 0, "top_p": 1.0}),
                   (RES, "test_all_equal_row_is_uniform_and_minus_zero_ranks_below_plus_zero", {}),
                   (RES, "test_rows_are_keyed_by_global_row_id", {})],
}

# (name, part whose pins run, text to find (exactly once), replacement)
MUTANTS = [
    # Appendix A: entropy, log-probability, temperature scaling
    ("entropy: wrong sign of the W/S term", "entropy",
     "return log(st.S) - st.W / st.S;", "return log(st.S) + st.W / st.S;"),
    ("entropy: W loses its exponential factor", "entropy",
     "{ st.S += e; st.W += d * e; }", "{ st.S += e; st.W += d; }"),
    ("entropy: ln S dropped", "entropy",
     "return log(st.S) - st.W / st.S;", "return -st.W / st.S;"),
    ("logits multiplied by tau instead of divided (sum pass)", "entropy",
     "double d = load_logit(row, dtype, (size_t)i) / tau - st.m;",
     "double d = load_logit(row, dtype, (size_t)i) * tau - st.m * tau * tau;"),
    ("per-row temperature ignored", "entropy",
     "return tau_rows ? (double)tau_rows[r] : (double)tau_scalar;", "(void)tau_rows; (void)r; return (double)tau_scalar;"),
    ("training-side log-prob misses ln S", "entropy",
     "? load_logit(row, dtype, (size_t)t) / tau - st.m - log(st.S) : NAN;",
     "? load_logit(row, dtype, (size_t)t) / tau - st.m : NAN;"),
    ("bf16 widened by the wrong shift", "entropy",
     "(uint32_t)((const uint16_t *)base)[idx] << 16;", "(uint32_t)((const uint16_t *)base)[idx] << 15;"),
    ("row mask ignored in the batch entropy sum", "entropy",
     "if (!row_mask || row_mask[r]) { sum += entropy_out[r]; ++cnt; }", "{ sum += entropy_out[r]; ++cnt; }"),
    ("row stride ignored", "entropy",
     "const void *row = (const char *)logits + (size_t)r * (size_t)row_stride * esz;\n"
     "        double tau = row_tau(tau_rows, tau_scalar, r);\n"
     "        row_stats st = softmax_stats(row, dtype, V, tau);\n"
     "        entropy_out[r]",
     "const void *row = (const char *)logits + (size_t)r * (size_t)V * esz;\n"
     "        double tau = row_tau(tau_rows, tau_scalar, r);\n"
     "        row_stats st = softmax_stats(row, dtype, V, tau);\n"
     "        entropy_out[r]"),
    ("log-softmax: normaliser added instead of subtracted", "entropy",
     "out[i] = load_logit(row, dtype, (size_t)i) / tau - st.m - lnS;",
     "out[i] = load_logit(row, dtype, (size_t)i) / tau - st.m + lnS;"),
    ("rollout-side log-prob forgets the temperature", "sampling",
     "logp_out[r] = load_logit(row, dtype, (size_t)tok) / tau - st.m - log(st.S);",
     "logp_out[r] = load_logit(row, dtype, (size_t)tok) - st.m - log(st.S);"),
    # counter-based generator
    ("Philox: multipliers swapped", "rng",
     "uint64_t pa = M_A * (uint64_t)c0;", "uint64_t pa = M_B * (uint64_t)c0;"),
    ("Philox: Weyl constants swapped", "rng", "k0 += W_A; k1 += W_B;", "k0 += W_B; k1 += W_A;"),
    ("Philox: nine rounds", "rng", "round < 10; ++round", "round < 9; ++round"),
    ("Philox: output words permuted", "rng",
     "uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;", "uint32_t n0 = (uint32_t)(pb >> 32) ^ c3 ^ k0;"),
    ("noise: wrong word of the block", "rng", "return out[index & 3u];", "return out[(index + 1u) & 3u];"),
    ("noise: stream and row swapped in the counter", "rng",
     "{ index >> 2, (uint32_t)row, (uint32_t)(row >> 32), stream }",
     "{ index >> 2, stream, (uint32_t)(row >> 32), (uint32_t)row }"),
    ("uniform: 24 bits instead of 23", "rng", "((double)(word >> 9) + 0.5)", "((double)(word >> 8) + 0.5)"),
    ("Gumbel: sign", "rng", "return -log(-log(e3o_uniform(word)));", "return log(-log(e3o_uniform(word)));"),
    # two-level sampler
    ("sampler: level-1 score uses the mass, not its logarithm", "sampling",
     "double score = st.m + log(tile_mass[t])", "double score = st.m + tile_mass[t]"),
    ("sampler: level 2 draws from the tile stream", "sampling",
     "e3o_noise_word(seed, grow, 2u, (uint32_t)i)", "e3o_noise_word(seed, grow, 1u, (uint32_t)i)"),
    ("sampler: level 2 forgets the temperature", "sampling",
     "double score = load_logit(row, dtype, (size_t)i) / tau\n", "double score = load_logit(row, dtype, (size_t)i)\n"),
    ("sampler: tile ties go to the highest index", "sampling",
     "if (score > s1) { s2 = s1; s1 = score; best_tile = t; }", "if (score >= s1) { s2 = s1; s1 = score; best_tile = t; }"),
    ("sampler: column ties go to the highest index", "sampling",
     "if (score > c1) { c2 = c1; c1 = score; best_col = i; }", "if (score >= c1) { c2 = c1; c1 = score; best_col = i; }"),
    ("sampler: partition deals chunks by the wrong modulus", "sampling",
     "return (col / super) * lanes + (col % sweep) / chunk;", "return (col / super) * lanes + (col % super) / (chunk * depth);"),
    ("sampler: noise keyed by the local row", "sampling",
     "int32_t tok = sample_row(row, dtype, V, tau, st, seed, row_base + (uint64_t)r,",
     "int32_t tok = sample_row(row, dtype, V, tau, st, seed, (uint64_t)r,"),
    ("sampler: near-tie margin a thousand times tighter", "sampling",
     "return (s1 - s2) <= 1e-5 * scale;", "return (s1 - s2) <= 1e-8 * scale;"),
    # Eq. 2
    ("advantages: mean not subtracted", "advantages",
     "adv_out[i] = ((double)rewards[i] - mean) / (sigma + eps);", "adv_out[i] = ((double)rewards[i]) / (sigma + eps);"),
    ("advantages: variance instead of standard deviation", "advantages",
     "double sigma = sqrt(ss / (double)(n - ddof));", "double sigma = ss / (double)(n - ddof);"),
    ("advantages: ddof ignored", "advantages",
     "double sigma = sqrt(ss / (double)(n - ddof));", "double sigma = sqrt(ss / (double)n);"),
    ("advantages: identical rewards not special-cased", "advantages",
     "if (rmax == rmin) {", "if (0) {"),
    ("advantages: group boundary off by one", "advantages",
     "int64_t lo = group_offsets[g], hi = group_offsets[g + 1];\n        int64_t n = hi - lo;\n        if (n <= 0) continue;\n        double rmax",
     "int64_t lo = group_offsets[g], hi = group_offsets[g + 1] - 1;\n        int64_t n = hi - lo;\n        if (n <= 0) continue;\n        double rmax"),
    ("advantages: eps not added", "advantages",
     "adv_out[i] = ((double)rewards[i] - mean) / (sigma + eps);", "adv_out[i] = ((double)rewards[i] - mean) / sigma;"),
    # Eq. 4 / Eq. 5
    ("Eq. 4: lower clamp missing", "temperature", "if (next < tau_min) next = tau_min;\n    if (next > tau_max) next = tau_max;\n    *tau_next_out = next;\n    if (H_target_out) *H_target_out = target;\n    return 0;\n}\n\nint e3o_max_threads",
     "if (next > tau_max) next = tau_max;\n    *tau_next_out = next;\n    if (H_target_out) *H_target_out = target;\n    return 0;\n}\n\nint e3o_max_threads"),
    ("Eq. 4: two-entry vocabulary accepted", "temperature",
     "!(H_init > 0.0) || !isfinite(H_init) || vocab < 3 ||", "!(H_init > 0.0) || !isfinite(H_init) || vocab < 2 ||"),
    ("Eq. 5: annealing starts one step late", "temperature",
     "x = (double)(t - t_anneal) / (double)(t_max - t_anneal);", "x = (double)(t - t_anneal - 1) / (double)(t_max - t_anneal);"),
    ("Eq. 4: ln ln|V| dropped", "temperature",
     "log(alpha) / (lnV + log(lnV))", "log(alpha) / (lnV)"),
    ("Eq. 4: alpha inverted", "temperature", "double alpha = target / H_t;", "double alpha = H_t / target;"),
    ("Eq. 4: tau not squared", "temperature",
     "double next = tau_t * (1.0 + tau_t * log(alpha) / (lnV + log(lnV)));",
     "double next = tau_t * (1.0 + log(alpha) / (lnV + log(lnV)));"),
    ("Eq. 5: cosine term not halved", "temperature",
     "(eta + (1.0 - eta) * 0.5 * (1.0 + cos(pi * x)))", "(eta + (1.0 - eta) * (1.0 + cos(pi * x)))"),
    ("Eq. 5: progress measured from step 0", "temperature",
     "x = (double)(t - t_anneal) / (double)(t_max - t_anneal);", "x = (double)t / (double)t_max;"),
    # Section 4.1, Algorithm 1
    ("ranks: ascending instead of descending average reward", "budgets",
     "if (avg_j > avg_i || (avg_j == avg_i && j < i)) ++ahead;", "if (avg_j < avg_i || (avg_j == avg_i && j < i)) ++ahead;"),
    ("ranks: counted from zero", "budgets",
     "k_out[i] = (double)(ahead + 1) / (double)n;", "k_out[i] = (double)ahead / (double)n;"),
    ("Algorithm 1: proportional share rounded to nearest", "budgets",
     "(int64_t)floor((double)rem * k[i] / sum_k);", "(int64_t)floor((double)rem * k[i] / sum_k + 0.5);"),
    ("Algorithm 1: leftovers go to the easiest first", "budgets",
     "if (k[x] > k[y] || (k[x] == k[y] && x < y)) best = b;", "if (k[x] < k[y] || (k[x] == k[y] && x < y)) best = b;"),
    ("Algorithm 1: G_max not enforced in the proportional step", "budgets",
     "if (g > G_max) g = G_max;\n        G_out[i] = (int32_t)g;", "G_out[i] = (int32_t)g;"),
    ("bounds: both move up", "budgets",
     "int64_t lo = (int64_t)G - (int64_t)step * passes_done;", "int64_t lo = (int64_t)G + (int64_t)step * passes_done;"),
    ("Algorithm 1: greedy pass ignores G_max", "budgets",
     "if (G_out[i] < G_max) { G_out[i] += 1; left -= 1; }", "{ G_out[i] += 1; left -= 1; }"),
    ("ranks: ties broken by the higher index", "budgets",
     "if (avg_j > avg_i || (avg_j == avg_i && j < i)) ++ahead;", "if (avg_j > avg_i || (avg_j == avg_i && j > i)) ++ahead;"),
    ("ranks: unseen questions rank as easiest", "budgets",
     "double avg_i = cum_rollouts[i] > 0 ? cum_reward[i] / (double)cum_rollouts[i] : 0.0;",
     "double avg_i = cum_rollouts[i] > 0 ? cum_reward[i] / (double)cum_rollouts[i] : 1e30;"),
    # Appendix A's measured gap
    ("gap update: alpha inverted", "gap",
     "double next = tau_t * (1.0 + tau_t * log(target / H_t) / delta);",
     "double next = tau_t * (1.0 + tau_t * log(H_t / target) / delta);"),
    ("gap: the maximum is not excluded", "gap", "if (i == imax) continue;", ""),
    ("gap: unweighted mean", "gap", "weighted += gap * e;", "weighted += gap; e = 1.0;"),
    ("gap update: Delta multiplies", "gap",
     "double next = tau_t * (1.0 + tau_t * log(target / H_t) / delta);",
     "double next = tau_t * (1.0 + tau_t * log(target / H_t) * delta);"),
    # Eq. 1
    ("objective: max instead of min", "objective", "double term = a < b ? a : b;", "double term = a > b ? a : b;"),
    ("objective: clip window one-sided", "objective",
     "double rc = r < 1.0 - clip_eps ? 1.0 - clip_eps : (r > 1.0 + clip_eps ? 1.0 + clip_eps : r);",
     "double rc = r > 1.0 + clip_eps ? 1.0 + clip_eps : r;"),
    ("objective: ratio inverted", "objective",
     "double r = exp((double)logp_new[t] - (double)logp_old[t]);", "double r = exp((double)logp_old[t] - (double)logp_new[t]);"),
    ("objective: token mean replaced by a sum", "objective",
     "double seq_mean = t1 > t0 ? seq_sum / (double)(t1 - t0) : 0.0;", "double seq_mean = seq_sum;"),
    ("objective: empty groups leave the mean over questions", "objective",
     "*objective_out = num_groups > 0 ? total / (double)num_groups : 0.0;",
     "{ int nz = 0; for (int32_t q = 0; q < num_groups; ++q) nz += group_offsets[q + 1] > group_offsets[q];\n"
     "      *objective_out = nz > 0 ? total / (double)nz : 0.0; }"),
    ("objective: group mean replaced by a sum", "objective",
     "if (i1 > i0) total += group_sum / (double)(i1 - i0);", "if (i1 > i0) total += group_sum;"),
    # restricted sampling
    ("restricted: race noise indexed by the rank instead of the bit pattern", "restricted",
     "e3o_noise_word(seed, grow, 3u, it[lv_first[j]].bits)", "e3o_noise_word(seed, grow, 3u, (uint32_t)j)"),
    ("restricted: race mass forgets the multiplicity", "restricted",
     "double mass = (double)(LV_END(j) - lv_first[j]) * exp((z - z1) / tau);", "double mass = exp((z - z1) / tau);"),
    ("restricted: position scaled by the wrong power of two", "restricted",
     "int64_t pos = (int64_t)(((2u * k23 + 1u) * (uint64_t)n) >> 24);", "int64_t pos = (int64_t)(((2u * k23 + 1u) * (uint64_t)n) >> 25);"),
    ("restricted: kept count one level short", "restricted",
     "if (kept_out) kept_out[r] = (int32_t)LV_END(jp);", "if (kept_out) kept_out[r] = (int32_t)lv_first[jp];"),
    ("restricted: levels ranked lowest first", "restricted",
     "if (a->ord != b->ord) return a->ord > b->ord ? -1 : 1;", "if (a->ord != b->ord) return a->ord < b->ord ? -1 : 1;"),
    ("top-k: one level too many", "restricted",
     "while (LV_END(jk) < (int64_t)top_k) ++jk;", "while (LV_END(jk) <= (int64_t)top_k) ++jk;"),
    ("top-p: threshold against the whole row instead of the top-k set", "restricted",
     "double T = top_p * lv_M[jk];", "double T = top_p * lv_M[nlev - 1];"),
    ("top-p: stops one level early", "restricted",
     "while (jp < jk && !(lv_M[jp] >= T)) ++jp;", "while (jp < jk && !(lv_M[jp + 1] >= T)) ++jp;"),
    ("restricted: log-prob normalised by the whole row", "restricted",
     "/ tau - log(lv_M[jp]);", "/ tau - log(lv_M[nlev - 1]);"),
    ("restricted: -0 ranks above +0", "restricted",
     "return (f32bits & 0x80000000u) ? ~f32bits : (f32bits | 0x80000000u);",
     "return (f32bits & 0x7FFFFFFFu) == 0 ? ((f32bits >> 31) ? 0x80000001u : 0x80000000u)\n"
     "         : ((f32bits & 0x80000000u) ? ~f32bits : (f32bits | 0x80000000u));"),
    ("restricted: level weight forgets the multiplicity", "restricted",
     "M += (double)(e - i) * exp((z - z1) / tau);", "M += exp((z - z1) / tau);"),
]


def _build(tmp_path, tag: str, text: str) -> ctypes.CDLL:
    src = tmp_path / f"oracle_{tag}.c"
    lib = tmp_path / f"liboracle_{tag}.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-w",
                    "-o", str(lib), str(src), "-lm"], check=True)
    L = ctypes.CDLL(str(lib))
    o._declare(L)
    return L


def _run_pins(part: str):
    """Names of the pins of `part` that fail against whatever library the front end holds."""
    failed = []
    for module, func, kwargs in PINS[part]:
        fn = getattr(importlib.import_module(module), func)
        try:
            fn(**kwargs)
        except Exception as exc:                       # an assertion, or the front end refusing a result
            failed.append(f"{func}: {type(exc).__name__}")
    return failed


@pytest.fixture()
def swapped():
    real = o.lib()
    yield
    o._lib = real


def test_unmodified_source_passes_every_pin_used_here(tmp_path, swapped):
    o._lib = _build(tmp_path, "identity", open(SRC).read())
    for part in PINS:
        assert _run_pins(part) == [], part


@pytest.mark.parametrize("name,part,find,replace", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_noticed(name, part, find, replace, tmp_path, swapped):
    text = open(SRC).read()
    assert text.count(find) == 1, f"{name}: the text to mutate must occur exactly once"
    o._lib = _build(tmp_path, "mutant", text.replace(find, replace))
    failed = _run_pins(part)
    print(f"{name}: caught by {failed}")
    assert failed, f"no pin of '{part}' noticed: {name}"
