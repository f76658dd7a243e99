/*
 * CPU oracle for the E3 vocabulary pass, GRPO advantages and temperature update.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision
 * statement of what the HIP library must compute.  It shares no code with the
 * HIP path and nothing in the product may call it; only the tests, the smoke
 * check and the benchmark's CPU-baseline leg load it.
 *
 * Every function cites the passage of the paper (arXiv 2505.18573) it follows.
 * Where the paper leaves a point open (it never describes its sampler, nor says
 * which standard deviation Eq. 2 means) the reading taken is stated at the
 * function.  Loops are scalar and in the paper's order; the only parallelism is
 * an optional OpenMP split over independent rows, which changes no arithmetic.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define E3O_F32 0
#define E3O_BF16 1

/* ------------------------------------------------------------------------ */
/* Stored logit -> double.  bf16 is the upper half of an IEEE binary32, so   */
/* widening is exact.                                                         */
/* ------------------------------------------------------------------------ */
static double load_logit(const void *base, int dtype, size_t idx)
{
    if (dtype == E3O_F32)
        return (double)((const float *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------------ */
/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random   */
/* numbers: as easy as 1, 2, 3", SC'11, Section 3.3 and Table 2 constants).   */
/* One round: two 32x32->64 products; the high halves are xored with the      */
/* other counter words and the round key, the low halves pass through.  The   */
/* key is bumped by the Weyl constants between rounds.                        */
/* ------------------------------------------------------------------------ */
void e3o_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M_A = 0xD2511F53u, M_B = 0xCD9E8D57u;
    const uint32_t W_A = 0x9E3779B9u, W_B = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t pa = M_A * (uint64_t)c0;
        uint64_t pb = M_B * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)pb;
        uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)pa;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W_A; k1 += W_B;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * Noise addressing (the paper does not describe its sampler; this is the
 * library's definition).  key = (seed low, seed high); counter =
 * (index / 4, row low, row high, stream); the word used is out[index % 4].
 * stream 1 indexes tiles, stream 2 indexes columns.  `row` is the global row
 * id, so a result does not depend on how rows are batched.
 */
uint32_t e3o_noise_word(uint64_t seed, uint64_t row, uint32_t stream, uint32_t index)
{
    uint32_t ctr[4] = { index >> 2, (uint32_t)row, (uint32_t)(row >> 32), stream };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    e3o_philox4x32_10(ctr, key, out);
    return out[index & 3u];
}

/* 23 random bits -> u = (k + 1/2) 2^-23, strictly inside (0,1). */
double e3o_uniform(uint32_t word)
{
    return ((double)(word >> 9) + 0.5) * (1.0 / 8388608.0);
}

/* Standard Gumbel variate g = -ln(-ln u). */
double e3o_gumbel(uint32_t word)
{
    return -log(-log(e3o_uniform(word)));
}

/* ------------------------------------------------------------------------ */
/* Column partition used by the two-level sampler.  A chunk is `chunk`        */
/* consecutive columns; chunks are dealt round-robin to `lanes` slots; a tile  */
/* is `depth` successive chunks of one slot.  (chunk,lanes,depth)=(c,1,d)      */
/* gives contiguous tiles of c*d columns; (1,1,1) makes every column a tile.   */
/* ------------------------------------------------------------------------ */
static int64_t tile_of(int64_t col, int64_t chunk, int64_t lanes, int64_t depth)
{
    int64_t sweep = chunk * lanes;          /* columns per round-robin sweep */
    int64_t super = sweep * depth;          /* columns per group of `lanes` tiles */
    return (col / super) * lanes + (col % sweep) / chunk;
}

int64_t e3o_num_tiles(int64_t V, int64_t chunk, int64_t lanes, int64_t depth)
{
    int64_t super = chunk * lanes * depth;
    return ((V + super - 1) / super) * lanes;
}

int64_t e3o_tile_of(int64_t col, int64_t chunk, int64_t lanes, int64_t depth)
{
    return tile_of(col, chunk, lanes, depth);
}

/* ------------------------------------------------------------------------ */
/* Softmax statistics of one row at temperature tau (Appendix A: p_i =        */
/* exp(z_i/tau)/sum_j exp(z_j/tau), written in max-shifted form with          */
/* Delta_i = z_max - z_i, beta = 1/tau, Z(beta) = sum_j exp(-beta Delta_j)).   */
/* m = max_i a_i, S = Z = sum exp(a_i - m), W = sum (a_i - m) exp(a_i - m).    */
/* A term whose exponential underflows to 0 contributes exactly 0.            */
/* ------------------------------------------------------------------------ */
typedef struct { double m, S, W; } row_stats;

static row_stats softmax_stats(const void *row, int dtype, int64_t V, double tau)
{
    row_stats st;
    st.m = -INFINITY;
    for (int64_t i = 0; i < V; ++i) {
        double a = load_logit(row, dtype, (size_t)i) / tau;
        if (a > st.m) st.m = a;
    }
    st.S = 0.0; st.W = 0.0;
    for (int64_t i = 0; i < V; ++i) {
        double d = load_logit(row, dtype, (size_t)i) / tau - st.m;
        double e = exp(d);
        if (e > 0.0) { st.S += e; st.W += d * e; }
    }
    return st;
}

/* Entropy via the Appendix-A decomposition H = beta sum p_i Delta_i + ln Z.
 * With the statistics above, beta sum p_i Delta_i = -W/S and Z = S. */
static double entropy_from_stats(row_stats st)
{
    return log(st.S) - st.W / st.S;
}

/* Shannon entropy written out from its definition (Eq. "entropy" in Appendix
 * A): H = -sum p_i ln p_i, skipping p_i = 0.  Used to cross-check the
 * decomposition inside the oracle's own tests. */
double e3o_entropy_textbook(const void *row, int dtype, int64_t V, double tau)
{
    double m = -INFINITY, Z = 0.0, H = 0.0;
    for (int64_t i = 0; i < V; ++i) {
        double a = load_logit(row, dtype, (size_t)i) / tau;
        if (a > m) m = a;
    }
    for (int64_t i = 0; i < V; ++i)
        Z += exp(load_logit(row, dtype, (size_t)i) / tau - m);
    for (int64_t i = 0; i < V; ++i) {
        double p = exp(load_logit(row, dtype, (size_t)i) / tau - m) / Z;
        if (p > 0.0) H -= p * log(p);
    }
    return H;
}

/* All V log-probabilities of one row: ln p_i = a_i - m - ln S. */
void e3o_log_softmax_row(const void *row, int dtype, int64_t V, double tau, double *out)
{
    row_stats st = softmax_stats(row, dtype, V, tau);
    double lnS = log(st.S);
    for (int64_t i = 0; i < V; ++i)
        out[i] = load_logit(row, dtype, (size_t)i) / tau - st.m - lnS;
}

/* Relative closeness test of the top two perturbed scores of a Gumbel-max
 * decision: rows that satisfy it are exempt from bit-exact token parity. */
static int near_tie(double s1, double s2)
{
    if (!(s2 > -INFINITY)) return 0;
    double scale = fmax(fmax(fabs(s1), fabs(s2)), 1.0);
    return (s1 - s2) <= 1e-5 * scale;
}

/*
 * Two-level Gumbel-max sample of one row.
 * Level 1: each tile T gets log-mass L_T = m + ln sum_{i in T} exp(a_i - m)
 * and one Gumbel g_T (stream 1, index = tile id); T* = argmax (L_T + g_T).
 * Level 2: inside T*, token = argmax_i (a_i + g_i) (stream 2, index = column).
 * By max-stability of the Gumbel law, max_{i in T}(a_i + g_i) ~ Gumbel(L_T)
 * independently of which i attains it, so P(token = i) = p_i exactly for any
 * partition.  Exact ties go to the lowest index at both levels.  A tile whose
 * mass underflows to 0 scores -inf and draws no noise.
 * diag (nullable): [s1_tile, s2_tile, s1_col, s2_col] = top-two scores.
 */
static int32_t sample_row(const void *row, int dtype, int64_t V, double tau, row_stats st,
                          uint64_t seed, uint64_t grow,
                          int64_t chunk, int64_t lanes, int64_t depth,
                          double *tile_mass, int64_t ntiles, uint8_t *tie_flag, double *diag)
{
    for (int64_t t = 0; t < ntiles; ++t) tile_mass[t] = 0.0;
    for (int64_t i = 0; i < V; ++i) {
        double e = exp(load_logit(row, dtype, (size_t)i) / tau - st.m);
        tile_mass[tile_of(i, chunk, lanes, depth)] += e;
    }
    double s1 = -INFINITY, s2 = -INFINITY;
    int64_t best_tile = -1;
    for (int64_t t = 0; t < ntiles; ++t) {
        if (!(tile_mass[t] > 0.0)) continue;
        double score = st.m + log(tile_mass[t])
                     + e3o_gumbel(e3o_noise_word(seed, grow, 1u, (uint32_t)t));
        if (score > s1) { s2 = s1; s1 = score; best_tile = t; }
        else if (score > s2) s2 = score;
    }
    int flag = near_tie(s1, s2);
    if (diag) { diag[0] = s1; diag[1] = s2; }

    double c1 = -INFINITY, c2 = -INFINITY;
    int64_t best_col = -1;
    for (int64_t i = 0; i < V; ++i) {
        if (tile_of(i, chunk, lanes, depth) != best_tile) continue;
        double score = load_logit(row, dtype, (size_t)i) / tau
                     + e3o_gumbel(e3o_noise_word(seed, grow, 2u, (uint32_t)i));
        if (score > c1) { c2 = c1; c1 = score; best_col = i; }
        else if (score > c2) c2 = score;
    }
    flag |= near_tie(c1, c2);
    if (diag) { diag[2] = c1; diag[3] = c2; }
    *tie_flag = (uint8_t)flag;
    return (int32_t)best_col;
}

static double row_tau(const float *tau_rows, float tau_scalar, int64_t r)
{
    return tau_rows ? (double)tau_rows[r] : (double)tau_scalar;
}

/*
 * Rollout-side call: for every row, sample a token at temperature tau_r and
 * report its log-probability and the entropy of the tau-scaled distribution
 * (Section 5.1 fixes the temperature rollouts are drawn at; Appendix A softmax and entropy).
 * Outputs are double; near_tie_out and diag_out (4 doubles per row) nullable.
 * Returns 0, or -1 on allocation failure / bad arguments.
 */
int e3o_sample_entropy(const void *logits, int dtype, int64_t rows, int64_t V, int64_t row_stride,
                       const float *tau_rows, float tau_scalar,
                       uint64_t seed, uint64_t row_base,
                       int64_t chunk, int64_t lanes, int64_t depth,
                       int32_t *token_out, double *logp_out, double *entropy_out,
                       uint8_t *near_tie_out, double *diag_out, int nthreads)
{
    if (!logits || rows < 0 || V < 1 || (row_stride < V && row_stride != 0) ||
        chunk < 1 || lanes < 1 || depth < 1)
        return -1;   /* row_stride 0 = the same row for every r (different noise) */
    size_t esz = dtype == E3O_F32 ? 4 : 2;
    int64_t ntiles = e3o_num_tiles(V, chunk, lanes, depth);
    int failed = 0;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        double *mass = (double *)malloc((size_t)ntiles * sizeof(double));
        if (!mass) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        const void *row = (const char *)logits + (size_t)r * (size_t)row_stride * esz;
        double tau = row_tau(tau_rows, tau_scalar, r);
        row_stats st = softmax_stats(row, dtype, V, tau);
        uint8_t flag = 0;
        int32_t tok = sample_row(row, dtype, V, tau, st, seed, row_base + (uint64_t)r,
                                 chunk, lanes, depth, mass, ntiles, &flag,
                                 diag_out ? diag_out + 4 * r : NULL);
        token_out[r] = tok;
        if (entropy_out) entropy_out[r] = entropy_from_stats(st);
        if (logp_out)
            logp_out[r] = load_logit(row, dtype, (size_t)tok) / tau - st.m - log(st.S);
        if (near_tie_out) near_tie_out[r] = flag;
        free(mass);
    }
    return failed ? -1 : 0;
}

/*
 * Training-side call: log-probability of a given target token and the entropy
 * of every row, with logits divided by the temperature as in the forward pass
 * (end of the "Temperature Scheduler" paragraph, Section 4.2), plus the mean
 * entropy over the rows the mask keeps -- the H_t of Eq. 4 -- accumulated left
 * to right in double.  A target outside [0,V) gives logp = NaN.
 */
int e3o_logprob_entropy(const void *logits, int dtype, int64_t rows, int64_t V, int64_t row_stride,
                        const int32_t *target_ids, const uint8_t *row_mask,
                        const float *tau_rows, float tau_scalar,
                        double *logp_out, double *entropy_out,
                        double *entropy_sum_out, int64_t *entropy_count_out, int nthreads)
{
    if (!logits || rows < 0 || V < 1 || row_stride < V) return -1;
    size_t esz = dtype == E3O_F32 ? 4 : 2;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        const void *row = (const char *)logits + (size_t)r * (size_t)row_stride * esz;
        double tau = row_tau(tau_rows, tau_scalar, r);
        row_stats st = softmax_stats(row, dtype, V, tau);
        entropy_out[r] = entropy_from_stats(st);
        if (logp_out) {
            int32_t t = target_ids ? target_ids[r] : -1;
            logp_out[r] = (t >= 0 && t < V)
                ? load_logit(row, dtype, (size_t)t) / tau - st.m - log(st.S) : NAN;
        }
    }
    double sum = 0.0;
    int64_t cnt = 0;
    for (int64_t r = 0; r < rows; ++r)
        if (!row_mask || row_mask[r]) { sum += entropy_out[r]; ++cnt; }
    if (entropy_sum_out) *entropy_sum_out = sum;
    if (entropy_count_out) *entropy_count_out = cnt;
    return 0;
}

/*
 * Group-relative advantage, Eq. 2: A_i = (r_i - mean(r)) / std(r) over the
 * rollouts of one prompt.  Groups are stored CSR-style because the rollout
 * budget differs per prompt (Algorithm 1 returns a G_i per question).
 * Readings: std is the population one for ddof = 0 (the literal formula) and
 * Bessel-corrected for ddof = 1; when every reward of a group is identical the
 * advantage is zero (Section 4.2, second paragraph), decided by an exact
 * max == min test rather than by a computed sigma; eps (>= 0) is added to
 * sigma otherwise.  Empty groups write nothing.
 */
int e3o_grpo_advantages(const float *rewards, const int32_t *group_offsets, int32_t num_groups,
                        int32_t ddof, double eps, double *adv_out)
{
    if (num_groups < 0 || (ddof != 0 && ddof != 1)) return -1;
    for (int32_t g = 0; g < num_groups; ++g) {
        int64_t lo = group_offsets[g], hi = group_offsets[g + 1];
        int64_t n = hi - lo;
        if (n <= 0) continue;
        double rmax = rewards[lo], rmin = rewards[lo], sum = 0.0;
        for (int64_t i = lo; i < hi; ++i) {
            double r = rewards[i];
            if (r > rmax) rmax = r;
            if (r < rmin) rmin = r;
            sum += r;
        }
        if (rmax == rmin) {
            for (int64_t i = lo; i < hi; ++i) adv_out[i] = 0.0;
            continue;
        }
        double mean = sum / (double)n, ss = 0.0;
        for (int64_t i = lo; i < hi; ++i) {
            double d = (double)rewards[i] - mean;
            ss += d * d;
        }
        double sigma = sqrt(ss / (double)(n - ddof));
        for (int64_t i = lo; i < hi; ++i)
            adv_out[i] = ((double)rewards[i] - mean) / (sigma + eps);
    }
    return 0;
}

/*
 * Entropy target of step t: H_init before annealing starts, afterwards the
 * cosine schedule of Eq. 5, H_init [eta + (1-eta) (1 + cos(pi x))/2] with
 * x = (t - t_anneal)/(t_max - t_anneal).  Readings: x is clamped to [0,1];
 * t_max <= t_anneal with annealing on means x = 1; t_anneal < 0 switches
 * annealing off.
 */
double e3o_entropy_target(double H_init, int64_t t, int64_t t_anneal, int64_t t_max, double eta)
{
    if (t_anneal < 0 || t < t_anneal) return H_init;
    double x = 1.0;
    if (t_max > t_anneal) {
        x = (double)(t - t_anneal) / (double)(t_max - t_anneal);
        if (x < 0.0) x = 0.0;
        if (x > 1.0) x = 1.0;
    }
    const double pi = 3.14159265358979323846;
    return H_init * (eta + (1.0 - eta) * 0.5 * (1.0 + cos(pi * x)));
}


/* ------------------------------------------------------------------------ */
/* Restricted sampling: top-k and top-p (nucleus) truncation before the draw.  */
/* The paper samples its rollouts unrestricted (Section 5.1, temperature 1);   */
/* rollout engines usually offer both truncations, so this is the library's    */
/* definition, stated on value levels so that it does not depend on how equal  */
/* logits happen to be ordered:                                                */
/*   * a LEVEL is the set of columns that store one bit pattern; levels are    */
/*     ranked by stored value, highest first (-0 ranks just below +0);         */
/*     level j has n_j columns, value z_j and weight w_j = exp((z_j - z_1)/tau) */
/*   * C_j = n_1 + .. + n_j,  M_j = n_1 w_1 + .. + n_j w_j  (in that order)     */
/*   * top-k (k >= 1):  j_k = first j with C_j >= k  (ties at the cut are kept; */
/*     k = 0 or k >= V: all levels)                                            */
/*   * top-p (p < 1), applied to the distribution renormalised over the top-k  */
/*     levels:  j_p = first j <= j_k with M_j >= p M_{j_k};  p >= 1: j_p = j_k  */
/*   * the kept set is levels 1..j_p; the draw is a Gumbel-max in two steps:    */
/*       level:  argmax_j  ln(n_j w_j) + g_j, written as the race               */
/*               argmax_j n_j w_j / E_j with E_j = -ln u_j; u_j from stream 3,  */
/*               index = the level's stored bit pattern; ties to the higher level */
/*       column: the columns of a level are equally likely: with u from stream  */
/*               4, index 0, pos = floor(u n) = ((2k+1) n) >> 24 for            */
/*               u = (k + 1/2) 2^-23, and the token is the pos-th column of the */
/*               level in increasing column order                               */
/*   * logp = (z_tok - z_1)/tau - ln M_{j_p}  (log-probability under the        */
/*     truncated, renormalised distribution); kept = C_{j_p}.                   */
/* near_cut marks rows whose top-p threshold lies within 1e-9 (relative) of a   */
/* cumulative mass, near_tie rows whose two best race scores lie within 1e-5:   */
/* both are exempt from exact parity.                                           */
/* ------------------------------------------------------------------------ */
typedef struct { uint32_t ord; uint32_t bits; int32_t col; } level_item;

static int cmp_level_item(const void *pa, const void *pb)
{
    const level_item *a = (const level_item *)pa, *b = (const level_item *)pb;
    if (a->ord != b->ord) return a->ord > b->ord ? -1 : 1;      /* higher value first */
    return a->col < b->col ? -1 : (a->col > b->col ? 1 : 0);
}

/* monotone map of a binary32 pattern to an unsigned integer (value order, -0 < +0) */
static uint32_t order_key(uint32_t f32bits)
{
    return (f32bits & 0x80000000u) ? ~f32bits : (f32bits | 0x80000000u);
}

int e3o_sample_restricted(const void *logits, int dtype, int64_t rows, int64_t V, int64_t row_stride,
                          const float *tau_rows, float tau_scalar, int32_t top_k, double top_p,
                          uint64_t seed, uint64_t row_base,
                          int32_t *token_out, double *logp_out, int32_t *kept_out,
                          uint8_t *near_tie_out, uint8_t *near_cut_out, int nthreads)
{
    if (!logits || rows < 0 || V < 1 || V > 0x7fffffff || (row_stride < V && row_stride != 0) ||
        top_k < 0 || !(top_p > 0.0))
        return -1;
    size_t esz = dtype == E3O_F32 ? 4 : 2;
    int failed = 0;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        level_item *it = (level_item *)malloc((size_t)V * sizeof(level_item));
        int64_t *lv_first = (int64_t *)malloc((size_t)V * sizeof(int64_t));   /* first item of level j */
        double *lv_M = (double *)malloc((size_t)V * sizeof(double));
        if (!it || !lv_first || !lv_M) {
#pragma omp atomic write
            failed = 1;
            free(it); free(lv_first); free(lv_M);
            continue;
        }
        const void *row = (const char *)logits + (size_t)r * (size_t)row_stride * esz;
        double tau = row_tau(tau_rows, tau_scalar, r);
        uint64_t grow = row_base + (uint64_t)r;
        for (int64_t i = 0; i < V; ++i) {
            uint32_t stored, as32;
            if (dtype == E3O_F32) { stored = ((const uint32_t *)row)[i]; as32 = stored; }
            else { stored = ((const uint16_t *)row)[i]; as32 = stored << 16; }
            it[i].ord = order_key(as32);
            it[i].bits = stored;
            it[i].col = (int32_t)i;
        }
        qsort(it, (size_t)V, sizeof(level_item), cmp_level_item);

        /* levels, cumulative counts and masses in rank order */
        double z1 = load_logit(row, dtype, (size_t)it[0].col);
        int64_t nlev = 0;
        double M = 0.0;
        for (int64_t i = 0; i < V; ) {
            int64_t e = i;
            while (e < V && it[e].ord == it[i].ord) ++e;
            double z = load_logit(row, dtype, (size_t)it[i].col);
            M += (double)(e - i) * exp((z - z1) / tau);
            lv_first[nlev] = i;
            lv_M[nlev] = M;
            ++nlev;
            i = e;
        }
        #define LV_END(j) ((j) + 1 < nlev ? lv_first[(j) + 1] : V)     /* C_j */
        int64_t jk = nlev - 1;
        if (top_k >= 1 && (int64_t)top_k < V) {
            jk = 0;
            while (LV_END(jk) < (int64_t)top_k) ++jk;
        }
        int64_t jp = jk;
        int cut_flag = 0;
        if (top_p < 1.0) {
            double T = top_p * lv_M[jk];
            jp = 0;
            while (jp < jk && !(lv_M[jp] >= T)) ++jp;
            double below = jp > 0 ? lv_M[jp - 1] : 0.0;
            if (T - below <= 1e-9 * T || lv_M[jp] - T <= 1e-9 * T) cut_flag = 1;
        }
        /* level race */
        double s1 = -INFINITY, s2 = -INFINITY;
        int64_t best = 0;
        for (int64_t j = 0; j <= jp; ++j) {
            double z = load_logit(row, dtype, (size_t)it[lv_first[j]].col);
            double mass = (double)(LV_END(j) - lv_first[j]) * exp((z - z1) / tau);   /* n_j w_j */
            double E = -log(e3o_uniform(e3o_noise_word(seed, grow, 3u, it[lv_first[j]].bits)));
            double q = mass / E;
            if (q > s1) { s2 = s1; s1 = q; best = j; }
            else if (q > s2) s2 = q;
        }
        int tie_flag = (s2 > 0.0) && (s1 - s2 <= 1e-5 * s1);
        /* column inside the level */
        int64_t n = LV_END(best) - lv_first[best];
        uint64_t k23 = (uint64_t)(e3o_noise_word(seed, grow, 4u, 0u) >> 9);
        int64_t pos = (int64_t)(((2u * k23 + 1u) * (uint64_t)n) >> 24);
        int32_t tok = it[lv_first[best] + pos].col;             /* items of a level are in column order */
        token_out[r] = tok;
        if (logp_out)
            logp_out[r] = (load_logit(row, dtype, (size_t)tok) - z1) / tau - log(lv_M[jp]);
        if (kept_out) kept_out[r] = (int32_t)LV_END(jp);
        if (near_tie_out) near_tie_out[r] = (uint8_t)tie_flag;
        if (near_cut_out) near_cut_out[r] = (uint8_t)cut_flag;
        #undef LV_END
        free(it); free(lv_first); free(lv_M);
    }
    return failed ? -1 : 0;
}

/*
 * Temperature update, Eq. 4: tau' = tau (1 + tau ln(alpha) / (ln|V| + ln ln|V|)),
 * alpha = H_target / H_t, H_target from e3o_entropy_target.  Readings: |V| is
 * the logit row width and must be >= 3 so that ln ln|V| exists; H_t, H_init,
 * tau must be finite and > 0 (else -5); the result is clamped to
 * [tau_min, tau_max]; (0, +inf) leaves Eq. 4 untouched; a non-positive factor
 * with tau_min = 0 is an error (-5).
 */
int e3o_temperature_update(double tau_t, double H_t, double H_init, int64_t vocab,
                           int64_t t, int64_t t_anneal, int64_t t_max, double eta,
                           double tau_min, double tau_max,
                           double *tau_next_out, double *H_target_out)
{
    if (!tau_next_out) return -1;
    if (!(tau_t > 0.0) || !isfinite(tau_t) || !(H_t > 0.0) || !isfinite(H_t) ||
        !(H_init > 0.0) || !isfinite(H_init) || vocab < 3 ||
        !(eta >= 0.0 && eta <= 1.0) || !(tau_min >= 0.0) || !(tau_max >= tau_min))
        return -5;
    double target = e3o_entropy_target(H_init, t, t_anneal, t_max, eta);
    if (!(target > 0.0)) return -5;
    double lnV = log((double)vocab);
    double alpha = target / H_t;
    double next = tau_t * (1.0 + tau_t * log(alpha) / (lnV + log(lnV)));
    if (!(next > 0.0) && !(tau_min > 0.0)) return -5;
    if (next < tau_min) next = tau_min;
    if (next > tau_max) next = tau_max;
    *tau_next_out = next;
    if (H_target_out) *H_target_out = target;
    return 0;
}

int e3o_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ======================================================================== */
/* Dynamic rollout budget (Section 4.1, Algorithm 1)                         */
/* ======================================================================== */

/*
 * Difficulty ranking, Section 4.1: questions are ranked by their average reward
 * r_c / n_c in descending order; k_i = rank(q_i) / |D|, rank counted from 1, so the
 * question with the lowest average reward gets k = 1 (hardest).  Readings: equal
 * averages keep their index order (the lower index ranks first); a question with no
 * rollouts yet counts as average reward 0.
 */
int e3o_difficulty_ranks(const double *cum_reward, const int64_t *cum_rollouts, int64_t n,
                         double *k_out)
{
    if (n < 0) return -2;
    for (int64_t i = 0; i < n; ++i) {
        if (cum_rollouts[i] < 0) return -5;
        double avg_i = cum_rollouts[i] > 0 ? cum_reward[i] / (double)cum_rollouts[i] : 0.0;
        if (!(avg_i == avg_i)) return -5;
        int64_t ahead = 0;                    /* questions that rank before i */
        for (int64_t j = 0; j < n; ++j) {
            if (j == i) continue;
            double avg_j = cum_rollouts[j] > 0 ? cum_reward[j] / (double)cum_rollouts[j] : 0.0;
            if (avg_j > avg_i || (avg_j == avg_i && j < i)) ++ahead;
        }
        k_out[i] = (double)(ahead + 1) / (double)n;
    }
    return 0;
}

/*
 * Algorithm 1.  N_total = B*G; every question starts at G_min; the remaining
 * N_total - B*G_min rollouts are split in proportion to k_i, rounded down; what the
 * rounding leaves over is handed out greedily in descending order of k, never above
 * G_max.  The batch total stays B*G.  Readings: the proportional step is capped at
 * G_max (the printed step can exceed it); "greedily" = passes over the questions in
 * descending k (ties: lower index first), one rollout per question per pass, skipping
 * those at G_max, until nothing is left.  Needs G_min <= G <= G_max, k_i finite >= 0
 * and sum k > 0.
 */
int e3o_allocate_budgets(const double *k, int32_t B, int32_t G, int32_t G_min, int32_t G_max,
                         int32_t *G_out)
{
    if (B < 0) return -2;
    if (G_min < 0 || G_min > G || G > G_max) return -5;
    if (B == 0) return 0;
    double sum_k = 0.0;
    for (int32_t i = 0; i < B; ++i) {
        if (!(k[i] >= 0.0) || !isfinite(k[i])) return -5;
        sum_k += k[i];
    }
    if (!(sum_k > 0.0)) return -5;
    int64_t total = (int64_t)B * G;
    int64_t rem = total - (int64_t)B * G_min;
    int64_t used = 0;
    for (int32_t i = 0; i < B; ++i) {
        int64_t extra = (int64_t)floor((double)rem * k[i] / sum_k);
        int64_t g = (int64_t)G_min + extra;
        if (g > G_max) g = G_max;
        G_out[i] = (int32_t)g;
        used += g;
    }
    int64_t left = total - used;
    /* order of descending k, ties by index: selection sort on an index array */
    int32_t *order = (int32_t *)malloc((size_t)B * sizeof(int32_t));
    if (!order) return -1;
    for (int32_t i = 0; i < B; ++i) order[i] = i;
    for (int32_t a = 0; a < B; ++a) {
        int32_t best = a;
        for (int32_t b = a + 1; b < B; ++b) {
            int32_t x = order[b], y = order[best];
            if (k[x] > k[y] || (k[x] == k[y] && x < y)) best = b;
        }
        int32_t t = order[a]; order[a] = order[best]; order[best] = t;
    }
    while (left > 0) {
        int64_t before = left;
        for (int32_t a = 0; a < B && left > 0; ++a) {
            int32_t i = order[a];
            if (G_out[i] < G_max) { G_out[i] += 1; left -= 1; }
        }
        if (left == before) break;             /* cannot happen while G <= G_max */
    }
    free(order);
    return left == 0 ? 0 : -5;
}

/*
 * Bounds curriculum (end of Section 4.1; Section 5.3 uses +-2 per pass over the
 * data): both bounds start at G; after each completed pass G_max grows and G_min
 * shrinks by `step` until they reach their limits.
 */
int e3o_budget_bounds(int32_t G, int32_t passes_done, int32_t step, int32_t G_min_limit,
                      int32_t G_max_limit, int32_t *G_min_out, int32_t *G_max_out)
{
    if (G < 0 || passes_done < 0 || step < 0 || G_min_limit < 0 || G_min_limit > G || G_max_limit < G)
        return -5;
    int64_t lo = (int64_t)G - (int64_t)step * passes_done;
    int64_t hi = (int64_t)G + (int64_t)step * passes_done;
    *G_min_out = (int32_t)(lo < G_min_limit ? G_min_limit : lo);
    *G_max_out = (int32_t)(hi > G_max_limit ? G_max_limit : hi);
    return 0;
}

/* ======================================================================== */
/* Logit gap Delta measured from the logits (Appendix A)                     */
/* ======================================================================== */

/*
 * Appendix A models a low-entropy row as one dominant logit z_max and all others a
 * common gap Delta below it, and notes that Delta could be estimated from the logits
 * (the paper then replaces it by ln N + ln ln N to avoid the extra pass).  Reading of
 * that remark, which comes without a formula: the probability-weighted mean gap of the
 * non-maximal tokens,
 *     Delta_hat = sum_{i != i*} p_i (z_max - z_i) / sum_{i != i*} p_i,
 * i* = the first index attaining the maximum, p = softmax(z / tau).  It equals Delta
 * exactly on the two-level model for every tau, and it is the quantity tied to the
 * entropy by the appendix's decomposition: H = beta (1 - p_max) Delta_hat + ln Z.
 * A row with a single column has no rest: Delta_hat = NaN.
 */
int e3o_logit_gaps(const void *logits, int dtype, int64_t rows, int64_t V, int64_t row_stride,
                   const float *tau_rows, float tau_scalar, double *gap_out)
{
    if (!logits || rows < 0 || V < 1 || (row_stride < V && row_stride != 0)) return -1;
    size_t esz = dtype == E3O_F32 ? 4 : 2;
    for (int64_t r = 0; r < rows; ++r) {
        const void *row = (const char *)logits + (size_t)r * (size_t)row_stride * esz;
        double tau = row_tau(tau_rows, tau_scalar, r);
        double zmax = -INFINITY;
        int64_t imax = 0;
        for (int64_t i = 0; i < V; ++i) {
            double z = load_logit(row, dtype, (size_t)i);
            if (z > zmax) { zmax = z; imax = i; }
        }
        double mass = 0.0, weighted = 0.0;
        for (int64_t i = 0; i < V; ++i) {
            if (i == imax) continue;
            double gap = zmax - load_logit(row, dtype, (size_t)i);
            double e = exp(-gap / tau);               /* p_i up to the common factor 1/Z */
            mass += e;
            weighted += gap * e;
        }
        gap_out[r] = mass > 0.0 ? weighted / mass : NAN;
    }
    return 0;
}

/*
 * Temperature update with a measured gap, Appendix A's relation before the
 * ln N + ln ln N substitution:  tau' = tau (1 + tau ln(alpha) / Delta),
 * alpha = H_target / H_t with the same target as Eq. 4 / Eq. 5.  Delta must be
 * finite and > 0; other guards as in e3o_temperature_update.
 */
int e3o_temperature_update_gap(double tau_t, double H_t, double H_init, double delta,
                               int64_t t, int64_t t_anneal, int64_t t_max, double eta,
                               double tau_min, double tau_max,
                               double *tau_next_out, double *H_target_out)
{
    if (!tau_next_out) return -1;
    if (!(tau_t > 0.0) || !isfinite(tau_t) || !(H_t > 0.0) || !isfinite(H_t) ||
        !(H_init > 0.0) || !isfinite(H_init) || !(delta > 0.0) || !isfinite(delta) ||
        !(eta >= 0.0 && eta <= 1.0) || !(tau_min >= 0.0) || !(tau_max >= tau_min))
        return -5;
    double target = e3o_entropy_target(H_init, t, t_anneal, t_max, eta);
    if (!(target > 0.0)) return -5;
    double next = tau_t * (1.0 + tau_t * log(target / H_t) / delta);
    if (!(next > 0.0) && !(tau_min > 0.0)) return -5;
    if (next < tau_min) next = tau_min;
    if (next > tau_max) next = tau_max;
    *tau_next_out = next;
    if (H_target_out) *H_target_out = target;
    return 0;
}

/* ======================================================================== */
/* GRPO clipped objective, Eq. 1 (forward value only)                        */
/* ======================================================================== */

/*
 * J = mean over questions q of (1/G_q) sum_{i in q} (1/|o_i|) sum_t
 *         min( r_{i,t} A_i , clip(r_{i,t}, 1-eps, 1+eps) A_i ),
 * r_{i,t} = pi_theta / pi_theta_old = exp(logp_new - logp_old) of token t of rollout i,
 * A_i the rollout's advantage (Eq. 2; the same for all its tokens).  The KL term of
 * Eq. 1 is dropped as in the paper (Section 3.1).  Rollouts are stored CSR-style
 * twice: seq_offsets[N+1] gives each rollout's token range, group_offsets[B+1] each
 * question's rollout range.  Readings: an empty rollout contributes 0; an empty group
 * contributes 0 and still counts in the mean over questions.
 * token_term_out [T] and seq_mean_out [N] are nullable.
 */
int e3o_grpo_objective(const float *logp_new, const float *logp_old, const int32_t *seq_offsets,
                       const float *adv, const int32_t *group_offsets, int32_t num_groups,
                       double clip_eps, double *token_term_out, double *seq_mean_out,
                       double *objective_out)
{
    if (num_groups < 0 || !(clip_eps >= 0.0)) return -5;
    double total = 0.0;
    for (int32_t q = 0; q < num_groups; ++q) {
        int32_t i0 = group_offsets[q], i1 = group_offsets[q + 1];
        double group_sum = 0.0;
        for (int32_t i = i0; i < i1; ++i) {
            int64_t t0 = seq_offsets[i], t1 = seq_offsets[i + 1];
            double A = (double)adv[i], seq_sum = 0.0;
            for (int64_t t = t0; t < t1; ++t) {
                double r = exp((double)logp_new[t] - (double)logp_old[t]);
                double rc = r < 1.0 - clip_eps ? 1.0 - clip_eps : (r > 1.0 + clip_eps ? 1.0 + clip_eps : r);
                double a = r * A, b = rc * A;
                double term = a < b ? a : b;
                if (token_term_out) token_term_out[t] = term;
                seq_sum += term;
            }
            double seq_mean = t1 > t0 ? seq_sum / (double)(t1 - t0) : 0.0;
            if (seq_mean_out) seq_mean_out[i] = seq_mean;
            group_sum += seq_mean;
        }
        if (i1 > i0) total += group_sum / (double)(i1 - i0);
    }
    *objective_out = num_groups > 0 ? total / (double)num_groups : 0.0;
    return 0;
}
