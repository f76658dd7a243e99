/*
 * libe3 -- the per-token vocabulary pass, group advantages and temperature
 * scheduler of "E3" (arXiv 2505.18573) for AMD MI355X (gfx950).
 *
 * C ABI: plain pointers and sizes only.  Unless a parameter says "host", every
 * pointer is DEVICE memory on the current HIP device.  The caller owns all
 * buffers; the library never retains a pointer.  Device entry points only
 * enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the
 * default stream) and return without synchronising: outputs are valid once the
 * stream has reached that point.  All argument checks happen on the host before
 * anything is launched; on error nothing is launched and outputs are untouched.
 * Results are bit-reproducible: the same call (same inputs, shapes and workspace
 * choice) gives the same bits in every run, since no floating-point atomics are
 * used and the order in which a row's columns are summed is fixed by the shape of
 * the launch.  A row that is part of a different batch (another number of rows, or
 * with / without a workspace) may run in a differently shaped launch: its token is
 * then the same except on near-ties, its entropy and log-prob the same up to fp32
 * rounding of the partial sums.
 *
 * Return value: 0 (E3_OK) or a negative e3_status.
 */
#ifndef E3_H
#define E3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    E3_OK = 0,
    E3_ERR_NULL = -1,      /* a required pointer is NULL */
    E3_ERR_SHAPE = -2,     /* rows < 0, V < 1, row_stride < V, num_groups < 0 ... */
    E3_ERR_DTYPE = -3,     /* dtype is not an e3_dtype */
    E3_ERR_ALIGN = -4,     /* logits base or row pitch not 16-byte aligned */
    E3_ERR_VALUE = -5,     /* a scalar is outside its domain (tau <= 0, H <= 0, ...) */
    E3_ERR_WORKSPACE = -6, /* e3_sample_entropy_noalloc only: more rows than its scratch serves */
    E3_ERR_LAUNCH = -7     /* the HIP runtime refused a launch (see hipGetLastError) */
} e3_status;

typedef enum { E3_F32 = 0, E3_BF16 = 1 } e3_dtype;

/*
 * Column partition of the two-level sampler (see e3_sample_entropy).  Columns
 * are cut into chunks of E3_TILE_CHUNK; chunks are dealt round-robin to
 * E3_TILE_LANES slots; a tile is E3_TILE_DEPTH successive chunks of one slot:
 *   tile(i) = (i / (CHUNK*LANES*DEPTH)) * LANES + (i % (CHUNK*LANES)) / CHUNK.
 * These constants are part of the definition of the sampled token and are frozen:
 * the token drawn for a given (seed, row, logits) never changes with a later
 * version of the kernels (tests/golden/sampler_tokens.txt holds stored tokens).
 */
#define E3_TILE_CHUNK 8
#define E3_TILE_LANES 64
#define E3_TILE_DEPTH 8

/* Static, never-freed description of a status code (host). */
const char* e3_strerror(int status);

/*
 * Bytes of device workspace that e3_sample_entropy / e3_logprob_entropy can use
 * for a [rows, V] problem (pure host function; 0 for rows > 1024, at most 2 MiB).
 * The workspace is optional: with it, a small batch (too few rows to give every
 * compute unit whole rows of its own) is cut into runs of columns that are streamed
 * by many workgroups, their 32-byte partial results staged in the workspace and
 * merged by a second launch on the same stream; without it, or when it is smaller
 * than this bound or not 16-byte aligned, every row is streamed by one workgroup,
 * which is correct for any shape but slow for small batches.  Both ways compute the
 * same quantities; tokens can differ between them only on rows whose sampling race
 * is decided within fp32 rounding (the rows the near-tie rule below exempts).
 * The workspace holds no state between calls; calls that share one must be ordered
 * (same stream) because the merge reads what the first launch wrote.
 */
size_t e3_workspace_bytes(int64_t rows, int64_t V);

/*
 * Rollout side: sample one token per row at temperature tau_r and report its
 * log-probability and the entropy of the tau-scaled distribution.
 *
 *   a_i = z_i / tau_r,  p_i = exp(a_i) / sum_j exp(a_j)      (Appendix A, softmax)
 *   H   = -sum_i p_i ln p_i                                   (Appendix A, entropy;
 *         evaluated as ln S - W/S, the appendix's decomposition
 *         H = beta sum p_i Delta_i + ln Z(beta) in max-shifted form)
 *   tok ~ p by two-level Gumbel-max (the paper samples "at temperature tau",
 *         Section 5.1, without describing a sampler; this is the library's):
 *         tile T* = argmax_T ( ln sum_{i in T} exp(a_i) + g_T ),
 *         tok     = argmax_{i in T*} ( a_i + g_i ),  g = -ln(-ln u),
 *         u = ((w >> 9) + 1/2) 2^-23, w = word (index % 4) of
 *         Philox4x32-10( counter = (index/4, row lo, row hi, stream),
 *                        key = (seed lo, seed hi) ),
 *         stream 1 / index = tile id for g_T, stream 2 / index = column for g_i,
 *         row = row_base + r.  Exact ties go to the lowest index.  By
 *         max-stability of the Gumbel law P(tok = i) = p_i exactly.
 *   logp = a_tok - ln sum_j exp(a_j)
 *
 * logits      [rows, row_stride] elements of `dtype`, row-major, first V of each
 *             row used; base 16-byte aligned and row_stride*sizeof(elem) a
 *             multiple of 16 (else E3_ERR_ALIGN).  Values must be finite; a row
 *             holding NaN or +-inf produces NaN outputs and an unspecified token
 *             in [0, V).
 * tau_rows    [rows] fp32 or NULL; when NULL tau_scalar (host, finite, > 0, else
 *             E3_ERR_VALUE) applies to every row.  Per-row values are not checked:
 *             a row with tau <= 0 produces NaN outputs.
 * seed, row_base  host scalars; row_base is the global id of row 0, so results do
 *             not depend on how rows are batched.
 * token_out   [rows] int32;  logp_out, entropy_out [rows] fp32 (natural log).
 *             logp_out and entropy_out may be NULL.
 * workspace   device scratch of workspace_bytes bytes, or NULL (see
 *             e3_workspace_bytes); contents on entry are ignored.
 * V           at most 1,040,384 columns (per-workgroup tables must fit LDS),
 *             else E3_ERR_SHAPE.
 * rows == 0 is a no-op.  fp32 accumulation per lane, fp64 merges.
 */
int e3_sample_entropy(const void* logits, int dtype, int64_t rows, int64_t V, int64_t row_stride,
                      const float* tau_rows, float tau_scalar,
                      uint64_t seed, uint64_t row_base,
                      int32_t* token_out, float* logp_out, float* entropy_out,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * e3_sample_entropy for callers that cannot allocate device memory and therefore cannot
 * bring the optional workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments (without the workspace pair), same
 * results bit for bit as e3_sample_entropy with a workspace of e3_workspace_bytes(rows, V):
 * the small-batch path stages its 32-byte row partials in a 2 MiB array that the library
 * holds in device memory for the life of the process (one copy per GPU it runs on, found
 * on this entry point's first call on that GPU).  The call allocates and frees nothing.
 *   rows  at most E3_NOALLOC_MAX_ROWS (what the array serves), else E3_ERR_WORKSPACE and
 *         nothing is launched; larger batches need no scratch at all: call
 *         e3_sample_entropy with workspace NULL.
 * All calls on one GPU share the array: calls that can overlap there (different streams,
 * different host threads) race on it and must be ordered by the caller; the array holds
 * no state between calls (every slot is written before it is read).
 */
#define E3_NOALLOC_MAX_ROWS 1024
int e3_sample_entropy_noalloc(const void* logits, int dtype, int64_t rows, int64_t V,
                              int64_t row_stride, const float* tau_rows, float tau_scalar,
                              uint64_t seed, uint64_t row_base,
                              int32_t* token_out, float* logp_out, float* entropy_out,
                              void* hip_stream);

/*
 * Rollout-side call with truncation: sample one token per row from the temperature-
 * scaled softmax restricted to the top-k and / or top-p (nucleus) part of the row.
 * The paper samples unrestricted (Section 5.1); this call covers the truncations that
 * rollout engines offer.  bf16 rows take every setting; fp32 rows need a count cut of
 * 1 <= top_k <= 256 (with or without top_p), anything else on fp32 rows is E3_ERR_VALUE.
 *
 * Definition (on value levels, so that it does not depend on the order of equal logits):
 *   a level is the set of columns storing one bit pattern; levels are ranked by value,
 *   highest first (-0 just below +0); level j has n_j columns and weight
 *   w_j = exp((z_j - z_1) / tau);  C_j = n_1 + .. + n_j,  M_j = n_1 w_1 + .. + n_j w_j.
 *   top_k >= 1: j_k = first j with C_j >= top_k (equal values at the cut are all kept);
 *               0, or >= V: no count cut.
 *   top_p < 1 : applied after top-k, to the distribution renormalised over levels
 *               1..j_k: j_p = first j <= j_k with M_j >= top_p * M_{j_k};  >= 1: j_p = j_k.
 *   The kept set is levels 1..j_p.  Draw: level = argmax_j n_j w_j / E_j with
 *   E_j = -ln u_j, u_j = uniform of Philox stream 3 at index = the level's bit pattern
 *   (same word -> uniform map as e3_sample_entropy; ties to the higher level); then
 *   with k the 23-bit integer of stream 4, index 0: pos = ((2k+1) n_j) >> 24 and the
 *   token is the pos-th column of the level in increasing column order.
 * Outputs: token_out [rows] int32; logp_out [rows] fp32 = ln of the token's probability
 *   under the truncated, renormalised distribution ((z_tok - z_1)/tau - ln M_{j_p});
 *   kept_out [rows] int32 = C_{j_p}.  logp_out and kept_out may be NULL.
 * Counts are exact; masses and the cuts are evaluated in fp64, the race scores in fp32.
 *   A row whose top_p target lies within 1e-9 (relative) of a cumulative mass may keep one
 *   level more or less than an fp64 reference with another summation order, and a row
 *   whose two best race scores lie within 1e-5 (relative) may draw the other level.
 * Logits must be finite (inf / NaN patterns are ignored as levels; a row without any
 *   finite logit gives token 0, logp NaN, kept 0).  Other arguments, alignment rules and
 *   errors as for e3_sample_entropy; top_k < 0 or top_p not in (0, inf): E3_ERR_VALUE.
 * One workgroup of 1024 threads per row.  With 1 <= top_k <= 256 the row is read once
 * (vector maxima kept in LDS, the few vectors that can hold one of the k largest read
 * again, exact selection among those); otherwise (bf16 only) a histogram over the 2^16
 * stored patterns in 128 KiB of LDS: one counting sweep of the row with 16-bit counters, or,
 * for a row with 65,536 or more equal columns, one to three sweeps with 32-bit counters.
 */
int e3_sample_restricted(const void* logits, int dtype, int64_t rows, int64_t V, int64_t row_stride,
                         const float* tau_rows, float tau_scalar, int32_t top_k, float top_p,
                         uint64_t seed, uint64_t row_base,
                         int32_t* token_out, float* logp_out, int32_t* kept_out, void* hip_stream);

/*
 * Training side: log-probability of a given token and the entropy of each row,
 * with the logits divided by the temperature as in the policy forward pass (end
 * of the "Temperature Scheduler" paragraph of Section 4.2), plus the two numbers
 * from which the batch-mean entropy H_t of Eq. 4 follows.
 *
 * target_ids  [rows] int32 or NULL; an id outside [0, V) gives logp = NaN.
 *             NULL requires logp_out == NULL.
 * row_mask    [rows] uint8 or NULL; rows with mask 0 (padding) are still written
 *             to logp_out/entropy_out but excluded from the batch sum.
 * logp_out    [rows] fp32 or NULL;  entropy_out [rows] fp32 (required).
 * entropy_sum_out    one double or NULL: sum of entropy_out over kept rows,
 *             accumulated in fp64 in a fixed order.
 * entropy_count_out  one int64 or NULL: number of kept rows.
 *             These two are each written once, by one plain store at the end of the
 *             last kernel, so they may also point into pinned host memory that the
 *             device can address (hipHostMalloc): the host then reads H_t's two
 *             numbers after waiting on an event recorded behind this call, without a
 *             copy in between.
 * Other arguments as for e3_sample_entropy.
 */
int e3_logprob_entropy(const void* logits, int dtype, int64_t rows, int64_t V, int64_t row_stride,
                       const int32_t* target_ids, const uint8_t* row_mask,
                       const float* tau_rows, float tau_scalar,
                       float* logp_out, float* entropy_out,
                       double* entropy_sum_out, int64_t* entropy_count_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * e3_logprob_entropy that also measures, in the same pass, the logit gap Delta of
 * Appendix A on every row: the paper's update is tau1 = tau0 (1 + tau0 ln(alpha) /
 * Delta) and it replaces Delta by ln N + ln ln N only because measuring it would cost
 * another pass over the logits; here it is a by-product of the sums already taken.
 *   gap_r = sum_{i != i*} p_i (z_max - z_i) / sum_{i != i*} p_i        (logit units)
 * with i* one index attaining the row maximum and p = softmax(z / tau_r); it equals
 * Delta exactly on the appendix's two-level model and satisfies the appendix's
 * decomposition H = beta (1 - p_max) gap + ln Z.  A one-column row gives NaN.
 * gap_out      [rows] fp32 or NULL.
 * gap_sum_out  one double (device) or NULL (needs gap_out): sum of gap_out over kept
 *              rows, fp64, fixed order.  count_out as entropy_count_out.
 */
int e3_logprob_entropy_gap(const void* logits, int dtype, int64_t rows, int64_t V, int64_t row_stride,
                           const int32_t* target_ids, const uint8_t* row_mask,
                           const float* tau_rows, float tau_scalar,
                           float* logp_out, float* entropy_out, float* gap_out,
                           double* entropy_sum_out, double* gap_sum_out, int64_t* count_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Group-relative advantage, Eq. 2:  A_i = (r_i - mean(r)) / std(r) over the
 * rollouts of one prompt, groups stored CSR-style because Algorithm 1 gives each
 * prompt its own rollout budget.
 *
 * rewards        [N] fp32, N = group_offsets[num_groups].
 * group_offsets  [num_groups + 1] int32, non-decreasing, group_offsets[0] = 0
 *                (caller's contract; not checked on the device).  Empty groups
 *                write nothing.
 * ddof           0 = population standard deviation (the literal formula),
 *                1 = Bessel-corrected.
 * eps            >= 0, added to the standard deviation.
 * adv_out        [N] fp32.  A group whose rewards are all identical (exact
 *                compare; includes groups of one) gets 0 for every rollout
 *                (Section 4.2: identical rewards give zero advantage).
 * Sums are taken in fp64.  num_groups == 0 is a no-op.
 */
int e3_grpo_advantages(const float* rewards, const int32_t* group_offsets,
                       int32_t num_groups, int32_t ddof, float eps,
                       float* adv_out, void* hip_stream);

/*
 * e3_logprob_entropy and e3_grpo_advantages in one call: the two sets of statistics a
 * GRPO update needs of a batch of finished rollouts (Eq. 2's advantages from the
 * rewards; log-probabilities and entropies from the logits, Section 4.2).  Results are
 * bit for bit those of the two separate calls.  When the batch runs as whole rows per
 * workgroup and there are at most as many groups as workgroups, the groups are computed
 * inside the vocabulary pass's launch by waves that have time to spare, which saves a
 * launch; otherwise they get a launch of their own first.  Arguments as for the two
 * calls; num_groups == 0 makes it e3_logprob_entropy.
 */
int e3_logprob_entropy_advantages(const void* logits, int dtype, int64_t rows, int64_t V,
                                  int64_t row_stride, const int32_t* target_ids,
                                  const uint8_t* row_mask, const float* tau_rows, float tau_scalar,
                                  float* logp_out, float* entropy_out,
                                  double* entropy_sum_out, int64_t* entropy_count_out,
                                  const float* rewards, const int32_t* group_offsets,
                                  int32_t num_groups, int32_t ddof, float eps, float* adv_out,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Forward value of the GRPO objective, Eq. 1 without the KL term (which the paper
 * drops, Section 3.1):
 *   J = mean_q (1/G_q) sum_{i in q} (1/|o_i|) sum_t min( r A_i , clip(r, 1-eps, 1+eps) A_i ),
 *   r = exp(logp_new[t] - logp_old[t]).
 * logp_new, logp_old  [T] fp32: log-probs of the rollout tokens under the current and
 *                     the sampling policy (e3_logprob_entropy / e3_sample_entropy).
 * seq_offsets    [num_seqs + 1] int32: token range of each rollout (CSR).
 * adv            [num_seqs] fp32: per-rollout advantage (e3_grpo_advantages).
 * group_offsets  [num_groups + 1] int32: rollout range of each question (CSR; the
 *                same array e3_grpo_advantages takes).  group_offsets[num_groups]
 *                must equal num_seqs (caller's contract).
 * clip_eps       >= 0 (E3_ERR_VALUE otherwise).
 * token_term_out [T] fp32 or NULL: the per-token min(...) term.
 * seq_mean_out   [num_seqs] fp64, required: per-rollout mean term (0 for an empty
 *                rollout); also the staging buffer of the two-stage reduction.
 * objective_out  one double (device), required.  An empty group contributes 0 and
 *                still counts in the mean over questions; num_groups == 0 gives 0.
 * Sums in fp64 in a fixed order.
 */
int e3_grpo_objective(const float* logp_new, const float* logp_old, const int32_t* seq_offsets,
                      const float* adv, int32_t num_seqs, const int32_t* group_offsets,
                      int32_t num_groups, float clip_eps, float* token_term_out,
                      double* seq_mean_out, double* objective_out, void* hip_stream);

/*
 * Temperature scheduler, host only (no GPU work, all pointers are HOST):
 *   H_target = H_init                                      for t < t_anneal or t_anneal < 0
 *            = H_init [eta + (1-eta)(1 + cos(pi x))/2]      otherwise (Eq. 5),
 *              x = clamp((t - t_anneal)/(t_max - t_anneal), 0, 1), x = 1 if t_max <= t_anneal
 *   alpha    = H_target / H_t
 *   tau_next = tau_t (1 + tau_t ln(alpha) / (ln|V| + ln ln|V|))               (Eq. 4)
 * then clamped to [tau_min, tau_max]; (0, +inf) leaves Eq. 4 untouched.
 * E3_ERR_VALUE if tau_t, H_t, H_init are not finite and > 0, vocab < 3, eta
 * outside [0,1], tau_min < 0, tau_max < tau_min, or the factor is <= 0 while
 * tau_min == 0.  On error the outputs are untouched.
 * tau_next_out required; H_target_out may be NULL.
 */
int e3_temperature_update(double tau_t, double H_t, double H_init, int64_t vocab,
                          int64_t t, int64_t t_anneal, int64_t t_max, double eta,
                          double tau_min, double tau_max,
                          double* tau_next_out, double* H_target_out);

/*
 * The same update with a measured gap instead of ln|V| + ln ln|V| (Appendix A, the
 * relation tau1 = tau0 (1 + tau0 ln(alpha) / Delta)); host only.  `gap` is the batch
 * mean of e3_logprob_entropy_gap's gap_out and must be finite and > 0; all else as
 * e3_temperature_update.
 */
int e3_temperature_update_gap(double tau_t, double H_t, double H_init, double gap,
                              int64_t t, int64_t t_anneal, int64_t t_max, double eta,
                              double tau_min, double tau_max,
                              double* tau_next_out, double* H_target_out);

/*
 * Difficulty ranking of the training questions, host only (Section 4.1): questions
 * are ranked by average reward cum_reward[i] / cum_rollouts[i] in descending order
 * and k_i = rank / num_questions, rank counted from 1, so the question answered worst
 * gets k = 1.  Equal averages rank in index order; a question with no rollouts yet
 * counts as average 0.  All pointers are HOST arrays of num_questions entries.
 * E3_ERR_VALUE for a negative rollout count or a NaN average.
 */
int e3_difficulty_ranks(const double* cum_reward, const int64_t* cum_rollouts,
                        int64_t num_questions, double* k_out);

/*
 * Algorithm 1 (Dynamic Rollout Budget), host only.  Given the normalised rankings
 * k[B] of a batch, the default budget G and the bounds G_min <= G <= G_max: every
 * question starts at G_min, the remaining B*G - B*G_min rollouts are split in
 * proportion to k_i (rounded down, capped at G_max), and what is left over is handed
 * out in passes over the questions in descending k (ties: lower index first), one
 * rollout per question per pass, skipping questions at G_max.  sum G_out = B*G.
 * G_out       [B] int32 (host).
 * offsets_out [B+1] int32 (host) or NULL: the CSR group offsets (prefix sums of
 *             G_out) in the form e3_grpo_advantages takes.
 * E3_ERR_VALUE unless G_min <= G <= G_max, k finite and >= 0 with a positive sum.
 */
int e3_allocate_budgets(const double* k, int32_t B, int32_t G, int32_t G_min, int32_t G_max,
                        int32_t* G_out, int32_t* offsets_out);

/*
 * Bounds curriculum, host only (end of Section 4.1): G_min and G_max start at G and
 * after each completed pass over the data move outwards by `step` until they reach
 * G_min_limit / G_max_limit (the paper's runs: G = 8, step 2, limits 4 and 12).
 */
int e3_budget_bounds(int32_t G, int32_t passes_done, int32_t step, int32_t G_min_limit,
                     int32_t G_max_limit, int32_t* G_min_out, int32_t* G_max_out);

#ifdef __cplusplus
}
#endif
#endif /* E3_H */
