// Restricted (top-k / top-p) sampling of bf16 logit rows for gfx950.
//
// Paper: arXiv 2505.18573 samples its rollouts unrestricted at temperature tau
// (Section 5.1); rollout engines usually offer both truncations, so the definition is
// the library's own and is stated in include/e3.h: columns that store one bit pattern
// form a LEVEL, levels are ranked by value, the cuts are taken on cumulative level
// counts (top-k) and cumulative level masses (top-p), and the draw is a Gumbel-max
// over the kept levels followed by a uniform choice among the winning level's columns.
//
// bf16 has only 65,536 bit patterns, so a row's whole value distribution fits a
// count histogram in the compute unit's 160 KiB LDS: all 65,536 patterns with 16-bit
// counters (128 KiB, two counters per word), or the 32,768 patterns of one sign with
// 32-bit counters (128 KiB).  One workgroup of 16 waves owns one row:
//   1. stream the row once, counting with LDS atomics (the columns of a wave
//      instruction scatter over many words: few conflicts);
//   2. every thread owns 64 (one window) or 32 (two windows) consecutive bins, i.e.
//      equally spaced values of one binade, whose weights exp((z - z_1)/tau) form a
//      geometric sequence: two exponentials and a product per bin give all level masses
//      in fp64; a workgroup scan yields the cumulative counts C_j and masses M_j in rank
//      order;
//   3. the cuts are located by the thread whose bins contain them, the kept levels
//      race for the draw (n_j w_j / E_j, fp32 like the unrestricted sampler), and a
//      second sweep over the row (now in L2 / the memory-side cache) finds the pos-th
//      column of the winning level.
// The one-window form (16-bit counters) serves every setting with that single counting
// sweep.  A row with a level of 65,536 or more equal columns wraps a counter; it is
// recognised (the counts no longer add up to the row's width) and redone by the
// two-window form: non-negative patterns first, and if the kept set reaches the negative
// patterns steps 1-2 again on the negative half (same LDS); there, top-p without top-k
// totals the negative half first, and the order of events "top-k cut among the
// negatives, top-p cut back among the non-negatives" costs a third sweep.  Counts are
// integers; masses and the cuts are fp64.
#include "vocab_common.h"
#include "vocab_pass.h"

namespace e3 {
namespace {

constexpr int kRThreads = 1024;
constexpr int kRWaves = kRThreads / 64;
constexpr int kBins = 32768;            // bit patterns of one sign
constexpr int kOwn = kBins / kRThreads; // 32 consecutive bins per thread
constexpr int kTrashBins = 64;          // words behind the window that take the other sign's patterns

struct RaceBest {
    double q;        // n_j w_j / E_j, -1 = none
    int bits;        // the level's stored bit pattern
    int n;           // its column count
};

struct Shared {
    double wave_M[kRWaves];
    int wave_C[kRWaves];
    float wave_top[kRWaves];
    double best_q[kRWaves];
    int best_bits[kRWaves];
    int best_n[kRWaves];
    int wave_hits[kRWaves];
    int wave_A[kRWaves];
    int first_thread;
    int cut_bin, cut_C;
    double cut_M;
    int token;
    int list_n;
    uint32_t list[1024];   // (vector index << 8 | 8-bit column mask) of vectors holding the winner
};
constexpr int kListCap = 1024;

__device__ __forceinline__ double bf16_value(int bits)
{
    return (double)__uint_as_float((uint32_t)bits << 16);
}

// Bin <-> bit pattern.  Non-negative window: bin = pattern.  Negative window:
// bin = 0xFFFF - pattern, so that in both windows a higher bin is a higher value.
__device__ __forceinline__ int bin_bits(bool hi, int bin) { return hi ? bin : 0xFFFF - bin; }

// Step 1: histogram of one sign's patterns over the whole row.
__device__ __forceinline__ void build_hist(const uint16_t* __restrict__ row, int64_t V, bool hi, uint32_t* hist, int tid)
{
    const uint4 zero4 = {0u, 0u, 0u, 0u};
    for (int i = tid; i < kBins / 4; i += kRThreads) reinterpret_cast<uint4*>(hist)[i] = zero4;
    __syncthreads();
    // bin = pattern (non-negative window) or 0xFFFF - pattern (negative window): one xor with a
    // uniform mask, done on the packed word for both halves.  A pattern of the other sign comes
    // out at 0x8000 or above and is counted into one of the kTrashBins words behind the window
    // (a word of the lane's own, so that the lanes of one instruction do not queue up on one
    // address): no branch, no lane masking around the LDS atomic.
    const uint32_t flip = hi ? 0u : 0xFFFFFFFFu;
    const uint32_t trash = (uint32_t)(kBins + (tid & (kTrashBins - 1)));
    auto add = [&](uint32_t bin) {                        // bin < 0x10000
        atomicAdd(&hist[bin < trash ? bin : trash], 1u);
    };
    auto add8 = [&](const u32x4& v) {
        const uint32_t x = v.x ^ flip, y = v.y ^ flip, z = v.z ^ flip, w = v.w ^ flip;
        add(x & 0xFFFFu); add(x >> 16); add(y & 0xFFFFu); add(y >> 16);
        add(z & 0xFFFFu); add(z >> 16); add(w & 0xFFFFu); add(w >> 16);
    };
    const int64_t nvec = V >> 3;
    const u32x4* rv = reinterpret_cast<const u32x4*>(row);
    int64_t v = tid;
    for (; v + 3 * kRThreads < nvec; v += 4 * kRThreads) {
        const u32x4 a = rv[v], b = rv[v + kRThreads], c = rv[v + 2 * kRThreads], d = rv[v + 3 * kRThreads];
        add8(a); add8(b); add8(c); add8(d);
    }
    for (; v < nvec; v += kRThreads) add8(rv[v]);
    const int64_t tail0 = nvec << 3;
    if (tid < V - tail0) add(((uint32_t)row[tail0 + tid] ^ flip) & 0xFFFFu);
    __syncthreads();
}

// Per-thread view of the scanned window.
template <int kOwnT>
struct ViewT {
    uint32_t cnt[kOwnT];  // counts of my bins; the last index is my highest bin
    int b0;               // my lowest bin
    double w_top, r_inv;  // weight of my highest bin; factor to the next lower bin
    int Cl, Cx;           // my count; count of all higher levels (carry included)
    double Ml, Mx;        // the same for mass
};
using View = ViewT<kOwn>;

// Step 2.  carry_C / carry_M: count and mass of all levels above this window.
// z1: value of the row's highest level; when `find_z1` it is taken from this window's
// highest populated bin (returns false if the window is empty).
__device__ __forceinline__ bool scan_window(const uint32_t* hist, bool hi, double inv_tau, bool find_z1, double& z1,
                            int carry_C, double carry_M, View& vw, int& Cw, double& Mw,
                            Shared& sh, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    vw.b0 = kBins - kOwn * (tid + 1);                 // thread 0 owns the highest bins
#pragma unroll
    for (int i = 0; i < kOwn / 4; ++i) {
        const uint4 c = reinterpret_cast<const uint4*>(hist + vw.b0)[i];
        vw.cnt[4 * i] = c.x; vw.cnt[4 * i + 1] = c.y; vw.cnt[4 * i + 2] = c.z; vw.cnt[4 * i + 3] = c.w;
    }
    const int top_bits_field = (bin_bits(hi, vw.b0 + kOwn - 1) >> 7) & 0xFF;
    const bool finite = top_bits_field != 0xFF;       // inf / NaN patterns are not levels
    int Cl = 0, my_top = -1;
#pragma unroll
    for (int j = 0; j < kOwn; ++j) {
        if (!finite) vw.cnt[j] = 0;
        Cl += (int)vw.cnt[j];
        if (vw.cnt[j] != 0) my_top = vw.b0 + j;
    }
    vw.Cl = Cl;
    if (find_z1) {
        const float t = wave_max((float)my_top);      // bins are below 2^15: exact in fp32
        if (lane == 0) sh.wave_top[wave] = t;
        __syncthreads();
        float top = -1.0f;
        for (int w = 0; w < kRWaves; ++w) top = fmaxf(top, sh.wave_top[w]);
        __syncthreads();
        if (top < 0.0f) { Cw = 0; Mw = 0.0; return false; }
        z1 = bf16_value(bin_bits(hi, (int)top));
    }
    // my 32 values are equally spaced (one binade, or the subnormals): geometric weights
    double Ml = 0.0;
    vw.w_top = 0.0; vw.r_inv = 0.0;
    if (Cl > 0) {
        const double z_top = bf16_value(bin_bits(hi, vw.b0 + kOwn - 1));
        const double step = ldexp(1.0, (top_bits_field ? top_bits_field : 1) - 134);
        vw.w_top = exp((z_top - z1) * inv_tau);
        vw.r_inv = exp(-step * inv_tau);
        double w = vw.w_top;
#pragma unroll
        for (int j = kOwn - 1; j >= 0; --j) {
            Ml += (double)vw.cnt[j] * w;
            w *= vw.r_inv;
        }
    }
    vw.Ml = Ml;
    // exclusive scan in thread order (= rank order)
    int Ci = Cl;
    double Mi = Ml;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int c = __shfl_up(Ci, d, 64);
        const double m = __shfl_up(Mi, d, 64);
        if (lane >= d) { Ci += c; Mi += m; }
    }
    if (lane == 63) { sh.wave_C[wave] = Ci; sh.wave_M[wave] = Mi; }
    __syncthreads();
    int Cb = carry_C;
    double Mb = carry_M;
    int Ct = 0;
    double Mt = 0.0;
    for (int w = 0; w < kRWaves; ++w) {
        if (w < wave) { Cb += sh.wave_C[w]; Mb += sh.wave_M[w]; }
        Ct += sh.wave_C[w]; Mt += sh.wave_M[w];
    }
    __syncthreads();
    vw.Cx = Cb + Ci - Cl;
    vw.Mx = Mb + (Mi - Ml);
    Cw = Ct; Mw = Mt;
    return true;
}

// First level whose cumulative count reaches k.  Exactly one thread holds it.
template <int kOwnT>
__device__ __forceinline__ void find_count_cut(const ViewT<kOwnT>& vw, int k, Shared& sh)
{
    if (vw.Cx < k && vw.Cx + vw.Cl >= k) {
        int C = vw.Cx;
        double M = vw.Mx, w = vw.w_top;
        int bin = vw.b0;
        bool done = false;
#pragma unroll
        for (int j = kOwnT - 1; j >= 0; --j) {
            if (!done) {
                C += (int)vw.cnt[j];
                M += (double)vw.cnt[j] * w;
                if (C >= k) { bin = vw.b0 + j; done = true; }
            }
            w *= vw.r_inv;
        }
        sh.cut_bin = bin; sh.cut_C = C; sh.cut_M = M;
    }
    __syncthreads();
}

// First level at or above `floor_bin` whose cumulative mass reaches T.  The scan's
// per-thread prefixes may disagree in the last bit, so the owner is the first thread
// whose inclusive prefix reaches T; if rounding lets none of its levels reach T the
// owner's lowest populated level (or the floor) is taken.
template <int kOwnT>
__device__ __forceinline__ void find_mass_cut(const ViewT<kOwnT>& vw, double T, int floor_bin, int floor_C, double floor_M,
                              Shared& sh, int tid)
{
    if (tid == 0) { sh.first_thread = kRThreads; }
    __syncthreads();
    if (vw.Cl > 0 && vw.Mx + vw.Ml >= T) atomicMin(&sh.first_thread, tid);
    __syncthreads();
    const int owner = sh.first_thread;
    if (owner == kRThreads) {                        // nobody reaches T: keep down to the floor
        if (tid == 0) { sh.cut_bin = floor_bin; sh.cut_C = floor_C; sh.cut_M = floor_M; }
    } else if (tid == owner) {
        int C = vw.Cx, bin = -1, Cb = 0;
        double M = vw.Mx, w = vw.w_top, Mb = 0.0;
        bool done = false;
#pragma unroll
        for (int j = kOwnT - 1; j >= 0; --j) {
            if (!done && vw.cnt[j] != 0) {
                C += (int)vw.cnt[j];
                M += (double)vw.cnt[j] * w;
                bin = vw.b0 + j; Cb = C; Mb = M;      // lowest populated level so far
                if (M >= T) done = true;
            }
            w *= vw.r_inv;
        }
        if (bin < floor_bin) { bin = floor_bin; Cb = floor_C; Mb = floor_M; }
        sh.cut_bin = bin; sh.cut_C = Cb; sh.cut_M = Mb;
    }
    __syncthreads();
}

// Race of the levels in bins [cut_bin, kBins) of the window in LDS: maximise
// n_j w_j / E_j with E_j = -ln u_j, u_j from Philox stream 3 at index = bit pattern.
// The scores are formed in fp32 (weights and variates as in the unrestricted sampler);
// decisions closer than fp32 resolves are the near-ties the parity rule exempts.
// Bins are dealt round-robin so that a short run of kept levels spreads over threads.
__device__ __forceinline__ RaceBest race_window(const uint32_t* hist, bool hi, int cut_bin, double z1,
                                                float c, uint64_t seed, uint64_t grow, RaceBest best,
                                                Shared& sh, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    const float z1f = (float)z1;                      // a bf16 value: exact
    RaceBest mine{-1.0, 0, 0};
    for (int bin = kBins - 1 - tid; bin >= cut_bin; bin -= kRThreads) {
        const uint32_t n = hist[bin];
        const int bits = bin_bits(hi, bin);
        if (n == 0 || ((bits >> 7) & 0xFF) == 0xFF) continue;
        uint32_t w4[4];
        philox4x32_10((uint32_t)bits >> 2, (uint32_t)grow, (uint32_t)(grow >> 32), 3u,
                      (uint32_t)seed, (uint32_t)(seed >> 32), w4);
        const int sel = bits & 3;
        const uint32_t word = sel == 0 ? w4[0] : sel == 1 ? w4[1] : sel == 2 ? w4[2] : w4[3];
        const float z = __uint_as_float((uint32_t)bits << 16);
        const float q = (float)n * __builtin_amdgcn_exp2f((z - z1f) * c) * inv_exp_variate(word);
        // a thread meets its bins in falling value order: `>` keeps the higher level on ties
        if ((double)q > mine.q) { mine.q = (double)q; mine.bits = bits; mine.n = (int)n; }
    }
    // workgroup argmax; ties to the higher value = higher bin of this window
    auto bin_of = [&](int bits) { return hi ? bits : 0xFFFF - bits; };
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const double oq = __shfl_xor(mine.q, d, 64);
        const int ob = __shfl_xor(mine.bits, d, 64);
        const int on = __shfl_xor(mine.n, d, 64);
        if (oq > mine.q || (oq == mine.q && oq >= 0.0 && bin_of(ob) > bin_of(mine.bits))) {
            mine.q = oq; mine.bits = ob; mine.n = on;
        }
    }
    if (lane == 0) { sh.best_q[wave] = mine.q; sh.best_bits[wave] = mine.bits; sh.best_n[wave] = mine.n; }
    __syncthreads();
    RaceBest out = best;                              // an earlier (higher) window wins ties
    bool from_here = false;
    for (int w = 0; w < kRWaves; ++w) {
        const double q = sh.best_q[w];
        if (q > out.q || (from_here && q == out.q && q >= 0.0 && bin_of(sh.best_bits[w]) > bin_of(out.bits))) {
            out.q = q; out.bits = sh.best_bits[w]; out.n = sh.best_n[w];
            from_here = true;
        }
    }
    __syncthreads();
    return out;
}

// ---------------------------------------------------------------------------
// One window.  All 65,536 patterns of a row counted in one sweep, two 16-bit counters per LDS
// word at the pattern's own index, so that one scan sees the whole row in rank order and no
// setting needs a second or third sweep.  A counter cannot hold a level of 65,536 columns or
// more: the counts of a row must add up to its width, a row where they do not (a wrapped
// counter changes the sum) is handed to the two-window code below, which counts in 32 bits.
// "Bin" here is the pattern's rank key, ascending in value: 0x8000 + pattern for non-negative
// patterns, 0xFFFF - pattern for negative ones; thread t owns the 64 bins below 65536 - 64 t,
// which are 64 consecutive patterns of one sign and one exponent.
// ---------------------------------------------------------------------------
constexpr int kBins1 = 65536;
constexpr int kOwn1 = kBins1 / kRThreads;          // 64

// A thread's share of the one window after the scan.  The counts themselves stay in LDS (64 of
// them per thread would occupy half the register file across the cut search); the one thread
// that holds a cut reads its own again.
struct ScanOne {
    int b0;               // my lowest bin
    bool finite;          // my patterns are values (not inf / NaN)
    double w_top, r_inv;  // weight of my highest bin; factor to the next lower bin
    int Cl, Cx;           // my count; count of all higher levels
    double Ml, Mx;        // the same for mass
};

__device__ __forceinline__ int bits_of_bin1(int bin) { return bin >= 0x8000 ? bin - 0x8000 : 0xFFFF - bin; }
__device__ __forceinline__ int bin1_of_bits(int bits) { return bits < 0x8000 ? bits + 0x8000 : 0xFFFF - bits; }
// Word that holds a pattern's counter.  One unused word follows every 32, so that the threads of
// a wave, each reading the 32 words of its 64 patterns, start in 64 different banks.
constexpr int kWords1 = kBins1 / 2 + kBins1 / 64;
__device__ __forceinline__ uint32_t word1(uint32_t bits) { return (bits >> 1) + (bits >> 6); }
__device__ __forceinline__ uint32_t count1(const uint32_t* hist, int bits)
{
    return (hist[word1((uint32_t)bits)] >> ((bits & 1) * 16)) & 0xFFFFu;
}

__device__ __forceinline__ void build_hist1(const uint16_t* __restrict__ row, int64_t V, uint32_t* hist, int tid)
{
    const uint4 zero4 = {0u, 0u, 0u, 0u};
    for (int i = tid; i < kWords1 / 4; i += kRThreads) reinterpret_cast<uint4*>(hist)[i] = zero4;
    __syncthreads();
    auto add2 = [&](uint32_t x) {                       // the two patterns of one word
        atomicAdd(&hist[word1(x & 0xFFFFu)], (x & 1u) ? 0x10000u : 1u);
        atomicAdd(&hist[word1(x >> 16)], (x & 0x10000u) ? 0x10000u : 1u);
    };
    auto add8 = [&](const u32x4& v) { add2(v.x); add2(v.y); add2(v.z); add2(v.w); };
    const int64_t nvec = V >> 3;
    const u32x4* rv = reinterpret_cast<const u32x4*>(row);
    int64_t v = tid;
    for (; v + 3 * kRThreads < nvec; v += 4 * kRThreads) {
        const u32x4 a = rv[v], b = rv[v + kRThreads], c = rv[v + 2 * kRThreads], d = rv[v + 3 * kRThreads];
        add8(a); add8(b); add8(c); add8(d);
    }
    for (; v < nvec; v += kRThreads) add8(rv[v]);
    const int64_t tail0 = nvec << 3;
    if (tid < V - tail0) {
        const uint32_t pat = row[tail0 + tid];
        atomicAdd(&hist[word1(pat)], (pat & 1u) ? 0x10000u : 1u);
    }
    __syncthreads();
}

// Scan of the one window.  Returns 0 if a counter has wrapped (the caller falls back), 1 if
// the row has no finite value, 2 otherwise, with z1 = the row's highest level, the window's
// count and mass in Cw / Mw and the thread's view filled in.
__device__ __forceinline__ int scan_one_window(const uint32_t* hist, int64_t V, double inv_tau, double& z1,
                                               ScanOne& vw, int& Cw, double& Mw, Shared& sh, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    vw.b0 = kBins1 - kOwn1 * (tid + 1);                // thread 0 owns the highest bins
    const bool nonneg = vw.b0 >= 0x8000;
    const int p_low = nonneg ? vw.b0 - 0x8000 : 0xFFFF - (vw.b0 + kOwn1 - 1);    // my lowest pattern, a multiple of 64
    const int exp_field = (p_low >> 7) & 0xFF;         // the same for all my patterns
    const bool finite = exp_field != 0xFF;             // inf / NaN patterns are not levels
    vw.finite = finite;
    int all = 0, Cl = 0, my_top = -1;
    uint32_t cnt[kOwn1];                               // in bin order; dead once my mass is summed
    // ascending bin = ascending pattern for non-negative values, descending for negative ones:
    // the negative half reads its words, and the two counters of a word, in reverse
#pragma unroll
    for (int i = 0; i < kOwn1 / 2; ++i) {
        const uint32_t word = hist[word1((uint32_t)p_low) + (nonneg ? i : kOwn1 / 2 - 1 - i)];
        const uint32_t lo = word & 0xFFFFu, hi = word >> 16;
        const uint32_t n0 = nonneg ? lo : hi, n1 = nonneg ? hi : lo;
        all += (int)(n0 + n1);
        cnt[2 * i] = finite ? n0 : 0u;
        cnt[2 * i + 1] = finite ? n1 : 0u;
        Cl += (int)(cnt[2 * i] + cnt[2 * i + 1]);
        if (cnt[2 * i] != 0) my_top = vw.b0 + 2 * i;
        if (cnt[2 * i + 1] != 0) my_top = vw.b0 + 2 * i + 1;
    }
    vw.Cl = Cl;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) all += __shfl_xor(all, d, 64);
    const float t = wave_max((float)my_top);           // bins are below 2^16: exact in fp32
    if (lane == 0) { sh.wave_top[wave] = t; sh.wave_A[wave] = all; }
    __syncthreads();
    float top = -1.0f;
    long long total = 0;
    for (int w = 0; w < kRWaves; ++w) { top = fmaxf(top, sh.wave_top[w]); total += sh.wave_A[w]; }
    __syncthreads();
    if (total != (long long)V) return 0;
    if (top < 0.0f) { Cw = 0; Mw = 0.0; return 1; }
    z1 = bf16_value(bits_of_bin1((int)top));
    // my 64 values are equally spaced (half a binade, or subnormals): geometric weights
    double Ml = 0.0;
    vw.w_top = 0.0; vw.r_inv = 0.0;
    if (Cl > 0) {
        const double z_top = bf16_value(bits_of_bin1(vw.b0 + kOwn1 - 1));
        const double step = ldexp(1.0, (exp_field ? exp_field : 1) - 134);
        vw.w_top = exp((z_top - z1) * inv_tau);
        vw.r_inv = exp(-step * inv_tau);
        double w = vw.w_top;
#pragma unroll
        for (int j = kOwn1 - 1; j >= 0; --j) {
            Ml += (double)cnt[j] * w;
            w *= vw.r_inv;
        }
    }
    vw.Ml = Ml;
    // exclusive scan in thread order (= rank order)
    int Ci = Cl;
    double Mi = Ml;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int c = __shfl_up(Ci, d, 64);
        const double m = __shfl_up(Mi, d, 64);
        if (lane >= d) { Ci += c; Mi += m; }
    }
    if (lane == 63) { sh.wave_C[wave] = Ci; sh.wave_M[wave] = Mi; }
    __syncthreads();
    int Cb = 0, Ct = 0;
    double Mb = 0.0, Mt = 0.0;
    for (int w = 0; w < kRWaves; ++w) {
        if (w < wave) { Cb += sh.wave_C[w]; Mb += sh.wave_M[w]; }
        Ct += sh.wave_C[w]; Mt += sh.wave_M[w];
    }
    __syncthreads();
    vw.Cx = Cb + Ci - Cl;
    vw.Mx = Mb + (Mi - Ml);
    Cw = Ct; Mw = Mt;
    return 2;
}

// The two cut searches of the one window: as find_count_cut / find_mass_cut, with the owner
// thread reading its counts from LDS again.
// The owner's 64 counts in bin order, read in one go (its 32 words are consecutive).
__device__ __forceinline__ void own_counts1(const uint32_t* hist, const ScanOne& vw, uint32_t cnt[kOwn1])
{
    const bool nonneg = vw.b0 >= 0x8000;
    const int p_low = nonneg ? vw.b0 - 0x8000 : 0xFFFF - (vw.b0 + kOwn1 - 1);
#pragma unroll
    for (int i = 0; i < kOwn1 / 2; ++i) {
        const uint32_t word = hist[word1((uint32_t)p_low) + (nonneg ? i : kOwn1 / 2 - 1 - i)];
        const uint32_t lo = word & 0xFFFFu, hi = word >> 16;
        cnt[2 * i] = vw.finite ? (nonneg ? lo : hi) : 0u;
        cnt[2 * i + 1] = vw.finite ? (nonneg ? hi : lo) : 0u;
    }
}

__device__ __forceinline__ void find_count_cut1(const uint32_t* hist, const ScanOne& vw, int k, Shared& sh)
{
    if (vw.Cx < k && vw.Cx + vw.Cl >= k) {
        int C = vw.Cx;
        double M = vw.Mx, w = vw.w_top;
        int bin = vw.b0;
        uint32_t cnt[kOwn1];
        own_counts1(hist, vw, cnt);
        bool done = false;
#pragma unroll
        for (int j = kOwn1 - 1; j >= 0; --j) {
            if (!done) {
                C += (int)cnt[j];
                M += (double)cnt[j] * w;
                if (C >= k) { bin = vw.b0 + j; done = true; }
            }
            w *= vw.r_inv;
        }
        sh.cut_bin = bin; sh.cut_C = C; sh.cut_M = M;
    }
    __syncthreads();
}

__device__ __forceinline__ void find_mass_cut1(const uint32_t* hist, const ScanOne& vw, double T, int floor_bin,
                                               int floor_C, double floor_M, Shared& sh, int tid)
{
    if (tid == 0) { sh.first_thread = kRThreads; }
    __syncthreads();
    if (vw.Cl > 0 && vw.Mx + vw.Ml >= T) atomicMin(&sh.first_thread, tid);
    __syncthreads();
    const int owner = sh.first_thread;
    if (owner == kRThreads) {                        // nobody reaches T: keep down to the floor
        if (tid == 0) { sh.cut_bin = floor_bin; sh.cut_C = floor_C; sh.cut_M = floor_M; }
    } else if (tid == owner) {
        int C = vw.Cx, bin = -1, Cb = 0;
        double M = vw.Mx, w = vw.w_top, Mb = 0.0;
        uint32_t cnt[kOwn1];
        own_counts1(hist, vw, cnt);
        bool done = false;
#pragma unroll
        for (int j = kOwn1 - 1; j >= 0; --j) {
            if (!done && cnt[j] != 0) {
                C += (int)cnt[j];
                M += (double)cnt[j] * w;
                bin = vw.b0 + j; Cb = C; Mb = M;      // lowest populated level so far
                if (M >= T) done = true;
            }
            w *= vw.r_inv;
        }
        if (bin < floor_bin) { bin = floor_bin; Cb = floor_C; Mb = floor_M; }
        sh.cut_bin = bin; sh.cut_C = Cb; sh.cut_M = Mb;
    }
    __syncthreads();
}

// Race of the levels in bins [cut_bin, 65536) of the one window; same scores, same tie
// rule (the higher value) as race_window.
__device__ __forceinline__ RaceBest race_one_window(const uint32_t* hist, int cut_bin, double z1, float c,
                                                    uint64_t seed, uint64_t grow, Shared& sh, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    const float z1f = (float)z1;                      // a bf16 value: exact
    RaceBest mine{-1.0, 0, 0};
    for (int bin = kBins1 - 1 - tid; bin >= cut_bin; bin -= kRThreads) {
        const int bits = bits_of_bin1(bin);
        const uint32_t n = count1(hist, bits);
        if (n == 0 || ((bits >> 7) & 0xFF) == 0xFF) continue;
        uint32_t w4[4];
        philox4x32_10((uint32_t)bits >> 2, (uint32_t)grow, (uint32_t)(grow >> 32), 3u,
                      (uint32_t)seed, (uint32_t)(seed >> 32), w4);
        const int sel = bits & 3;
        const uint32_t word = sel == 0 ? w4[0] : sel == 1 ? w4[1] : sel == 2 ? w4[2] : w4[3];
        const float z = __uint_as_float((uint32_t)bits << 16);
        const float q = (float)n * __builtin_amdgcn_exp2f((z - z1f) * c) * inv_exp_variate(word);
        // a thread meets its bins in falling value order: `>` keeps the higher level on ties
        if ((double)q > mine.q) { mine.q = (double)q; mine.bits = bits; mine.n = (int)n; }
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const double oq = __shfl_xor(mine.q, d, 64);
        const int ob = __shfl_xor(mine.bits, d, 64);
        const int on = __shfl_xor(mine.n, d, 64);
        if (oq > mine.q || (oq == mine.q && oq >= 0.0 && bin1_of_bits(ob) > bin1_of_bits(mine.bits))) {
            mine.q = oq; mine.bits = ob; mine.n = on;
        }
    }
    if (lane == 0) { sh.best_q[wave] = mine.q; sh.best_bits[wave] = mine.bits; sh.best_n[wave] = mine.n; }
    __syncthreads();
    RaceBest out{-1.0, 0, 0};
    for (int w = 0; w < kRWaves; ++w) {
        const double q = sh.best_q[w];
        if (q > out.q || (q == out.q && q >= 0.0 && bin1_of_bits(sh.best_bits[w]) > bin1_of_bits(out.bits))) {
            out.q = q; out.bits = sh.best_bits[w]; out.n = sh.best_n[w];
        }
    }
    __syncthreads();
    return out;
}

// Step 3, last part, when the winning level has at most kListCap columns (the usual
// case): one pipelined sweep over the row in which every thread notes the vectors that
// hold the pattern in a short LDS list; the pos-th column in column order is then picked
// from the list by ranking its entries.
__device__ __forceinline__ int locate_listed(const uint16_t* __restrict__ row, int64_t V, int bits,
                                             int pos, Shared& sh, int tid)
{
    if (tid == 0) { sh.list_n = 0; sh.token = -1; }
    __syncthreads();
    const int64_t nvec = V >> 3;
    const u32x4* rv = reinterpret_cast<const u32x4*>(row);
    const uint32_t pat = (uint32_t)bits, pat2 = pat | (pat << 16);
    auto zero_half = [](uint32_t x) -> uint32_t { return (x - 0x00010001u) & ~x & 0x80008000u; };
    auto note = [&](int64_t v, const u32x4& t) {
        const uint32_t a = t.x ^ pat2, b = t.y ^ pat2, c = t.z ^ pat2, d = t.w ^ pat2;
        if ((zero_half(a) | zero_half(b) | zero_half(c) | zero_half(d)) != 0u) {
            uint32_t m = 0;
            m |= ((a & 0xFFFFu) == 0u) << 0; m |= ((a >> 16) == 0u) << 1;
            m |= ((b & 0xFFFFu) == 0u) << 2; m |= ((b >> 16) == 0u) << 3;
            m |= ((c & 0xFFFFu) == 0u) << 4; m |= ((c >> 16) == 0u) << 5;
            m |= ((d & 0xFFFFu) == 0u) << 6; m |= ((d >> 16) == 0u) << 7;
            if (m != 0u) {
                const int slot = atomicAdd(&sh.list_n, 1);
                if (slot < kListCap) sh.list[slot] = ((uint32_t)v << 8) | m;
            }
        }
    };
    const u32x4 filler = {~pat2, ~pat2, ~pat2, ~pat2};           // matches nothing
    for (int64_t v0 = tid; v0 < nvec; v0 += 8 * kRThreads) {
        u32x4 t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t vv = v0 + (int64_t)j * kRThreads;
            t[j] = vv < nvec ? rv[vv] : filler;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) note(v0 + (int64_t)j * kRThreads, t[j]);
    }
    if (tid == 0) {                                              // columns after the last whole vector
        uint32_t m = 0;
        for (int64_t c = nvec << 3; c < V; ++c)
            if ((uint32_t)row[c] == pat) m |= 1u << (int)(c - (nvec << 3));
        if (m != 0u) {
            const int slot = atomicAdd(&sh.list_n, 1);
            if (slot < kListCap) sh.list[slot] = ((uint32_t)nvec << 8) | m;
        }
    }
    __syncthreads();
    const int cnt = sh.list_n < kListCap ? sh.list_n : kListCap;
    if (tid < cnt) {
        const uint32_t mine = sh.list[tid];
        int rank = 0;
        for (int e = 0; e < cnt; ++e) {
            const uint32_t o = sh.list[e];
            if ((o >> 8) < (mine >> 8)) rank += __popc(o & 0xFFu);
        }
        const int here = __popc(mine & 0xFFu);
        if (pos >= rank && pos < rank + here) {
            uint32_t mm = mine & 0xFFu;
            for (int skip = pos - rank; skip > 0; --skip) mm &= mm - 1;   // drop the lowest set bits
            sh.token = (int)((mine >> 8) * 8u) + (__ffs(mm) - 1);
        }
    }
    __syncthreads();
    return sh.token;
}

// Step 3, last part, for levels of any size: the pos-th column (0-based, increasing
// column order) that stores `bits`, by counting.  Waves take contiguous runs of 16-byte vectors; the few columns past the last
// whole vector come last.
__device__ __forceinline__ int locate_column(const uint16_t* __restrict__ row, int64_t V, int bits, int pos,
                             Shared& sh, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t nvec = V >> 3;
    const int64_t per_wave = (nvec + kRWaves - 1) / kRWaves;
    const int64_t v_begin = (int64_t)wave * per_wave < nvec ? (int64_t)wave * per_wave : nvec;
    const int64_t v_end = v_begin + per_wave < nvec ? v_begin + per_wave : nvec;
    const u32x4* rv = reinterpret_cast<const u32x4*>(row);
    const uint32_t pat = (uint32_t)bits;
    auto mask_of = [&](const u32x4& v) -> uint32_t {
        uint32_t m = 0;
        m |= ((v.x & 0xFFFFu) == pat) << 0; m |= ((v.x >> 16) == pat) << 1;
        m |= ((v.y & 0xFFFFu) == pat) << 2; m |= ((v.y >> 16) == pat) << 3;
        m |= ((v.z & 0xFFFFu) == pat) << 4; m |= ((v.z >> 16) == pat) << 5;
        m |= ((v.w & 0xFFFFu) == pat) << 6; m |= ((v.w >> 16) == pat) << 7;
        return m;
    };
    // hits of my wave's run
    int hits = 0;
    for (int64_t v = v_begin + lane; v < v_end; v += 64) hits += __popc(mask_of(rv[v]));
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) hits += __shfl_xor(hits, d, 64);
    if (lane == 0) sh.wave_hits[wave] = hits;
    if (tid == 0) sh.token = -1;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += sh.wave_hits[w];
    int total = 0;
    for (int w = 0; w < kRWaves; ++w) total += sh.wave_hits[w];
    if (pos >= before && pos < before + hits) {       // uniform per wave: my run holds it
        int rem = pos - before;
        for (int64_t v0 = v_begin; v0 < v_end; v0 += 64) {
            const int64_t v = v0 + lane;
            const uint32_t m = v < v_end ? mask_of(rv[v]) : 0u;
            const int c = __popc(m);
            int inc = c;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int o = __shfl_up(inc, d, 64);
                if (lane >= d) inc += o;
            }
            const int sweep_total = __shfl(inc, 63, 64);
            if (rem < sweep_total) {
                if (rem >= inc - c && rem < inc) {    // exactly one lane
                    int skip = rem - (inc - c);
                    uint32_t mm = m;
                    while (skip-- > 0) mm &= mm - 1;  // drop the lowest set bits
                    sh.token = (int)(v * 8 + (__ffs(mm) - 1));
                }
                break;
            }
            rem -= sweep_total;
        }
    }
    // the columns after the last whole vector
    if (tid == 0 && pos >= total) {
        int rem = pos - total;
        for (int64_t c = nvec << 3; c < V; ++c)
            if ((uint32_t)row[c] == pat && rem-- == 0) { sh.token = (int)c; break; }
    }
    __syncthreads();
    return sh.token;
}

struct RestrictedArgs {
    const uint16_t* logits;
    int64_t rows, V, row_stride;
    const float* tau_rows;
    float tau_scalar;
    int32_t top_k;
    float top_p;
    uint64_t seed, row_base;
    int32_t* token_out;
    float* logp_out;
    int32_t* kept_out;
};

__global__ __launch_bounds__(kRThreads)
void sample_restricted_kernel(RestrictedArgs a)
{
    __shared__ __align__(16) uint32_t hist[kWords1 > kBins + kTrashBins ? kWords1 : kBins + kTrashBins];
    __shared__ Shared sh;
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    const int64_t V = a.V;
    const uint16_t* rowp = a.logits + row * a.row_stride;
    const float tau = a.tau_rows ? a.tau_rows[row] : a.tau_scalar;
    const double inv_tau = 1.0 / (double)tau;
    const float c = kLog2eF / tau;
    const uint64_t grow = a.row_base + (uint64_t)row;
    const bool k_on = a.top_k >= 1 && (int64_t)a.top_k < V;
    const bool p_on = a.top_p < 1.0f;
    const double p = (double)a.top_p;
    const int k = a.top_k;

    double z1 = 0.0;
    RaceBest best{-1.0, 0, 0};
    int kept_C = 0;
    double kept_M = 0.0;

    // One sweep, one scan, whatever the setting; rows with a level too long for a 16-bit
    // counter take the two-window code after it.
    bool done = false;
    {
        ScanOne v1;
        int C_all = 0;
        double M_all = 0.0;
        build_hist1(rowp, V, hist, tid);
        const int state = scan_one_window(hist, V, inv_tau, z1, v1, C_all, M_all, sh, tid);
        if (state != 0) {
            done = true;
            if (state == 2) {
                int cb = 0;
                kept_C = C_all; kept_M = M_all;
                if (k_on && C_all >= k) {
                    find_count_cut1(hist, v1, k, sh);
                    cb = sh.cut_bin; kept_C = sh.cut_C; kept_M = sh.cut_M;
                    __syncthreads();
                }
                if (p_on) {
                    find_mass_cut1(hist, v1, p * kept_M, cb, kept_C, kept_M, sh, tid);
                    cb = sh.cut_bin; kept_C = sh.cut_C; kept_M = sh.cut_M;
                    __syncthreads();
                }
                best = race_one_window(hist, cb, z1, c, a.seed, grow, sh, tid);
            }
        }
    }

    View vw;
    int C_hi = 0, C_lo = 0;
    double M_hi = 0.0, M_lo = 0.0;
    if (!done) {

    // Without top-k the nucleus target is a fraction of the whole row's mass, which
    // includes the negative patterns: total them first, relative to the value 0.
    double neg_mass_ref0 = 0.0;
    if (!k_on && p_on) {
        build_hist(rowp, V, false, hist, tid);
        double zero_ref = 0.0;
        int Cn;
        scan_window(hist, false, inv_tau, false, zero_ref, 0, 0.0, vw, Cn, neg_mass_ref0, sh, tid);
    }

    build_hist(rowp, V, true, hist, tid);
    const bool any_hi = scan_window(hist, true, inv_tau, true, z1, 0, 0.0, vw, C_hi, M_hi, sh, tid);

    // Does the kept set end inside the non-negative window?
    bool cut_in_hi = false;
    if (any_hi) {
        if (k_on) {
            if (C_hi >= k) {
                find_count_cut(vw, k, sh);
                const int kb = sh.cut_bin, kC = sh.cut_C;
                const double kM = sh.cut_M;
                __syncthreads();
                if (p_on) find_mass_cut(vw, p * kM, kb, kC, kM, sh, tid);
                cut_in_hi = true;
            }
        } else if (p_on) {
            const double T = p * (M_hi + neg_mass_ref0 * exp(-z1 * inv_tau));
            if (M_hi >= T) {
                find_mass_cut(vw, T, 0, C_hi, M_hi, sh, tid);
                cut_in_hi = true;
            }
        }
        if (cut_in_hi) {
            const int cb = sh.cut_bin;
            kept_C = sh.cut_C; kept_M = sh.cut_M;
            __syncthreads();
            best = race_window(hist, true, cb, z1, c, a.seed, grow, best, sh, tid);
        } else {
            best = race_window(hist, true, 0, z1, c, a.seed, grow, best, sh, tid);
            kept_C = C_hi; kept_M = M_hi;
        }
    }

    if (!cut_in_hi) {
        // The kept set reaches the negative patterns (or the row has no others).
        build_hist(rowp, V, false, hist, tid);
        const bool any_lo = scan_window(hist, false, inv_tau, !any_hi, z1, C_hi, M_hi, vw, C_lo, M_lo, sh, tid);
        if (any_lo) {
            int cb = 0;
            int cC = C_hi + C_lo;
            double cM = M_hi + M_lo;
            bool back_to_hi = false;
            if (k_on) {
                if (C_hi + C_lo >= k && C_hi < k) {
                    find_count_cut(vw, k, sh);
                    cb = sh.cut_bin; cC = sh.cut_C; cM = sh.cut_M;
                    __syncthreads();
                }
                if (p_on) {
                    const double T = p * cM;
                    if (any_hi && M_hi >= T) back_to_hi = true;       // nucleus ends above this window
                    else {
                        find_mass_cut(vw, T, cb, cC, cM, sh, tid);
                        cb = sh.cut_bin; cC = sh.cut_C; cM = sh.cut_M;
                        __syncthreads();
                    }
                }
            } else if (p_on) {
                const double T = p * (M_hi + M_lo);
                find_mass_cut(vw, T, 0, cC, cM, sh, tid);
                cb = sh.cut_bin; cC = sh.cut_C; cM = sh.cut_M;
                __syncthreads();
            }
            if (!back_to_hi) {
                best = race_window(hist, false, cb, z1, c, a.seed, grow, best, sh, tid);
                kept_C = cC; kept_M = cM;
            } else {
                // third sweep: the top-k cut lies among the negatives, the nucleus of that
                // set ends among the non-negatives
                const double T = p * cM;
                int Cd; double Md;
                build_hist(rowp, V, true, hist, tid);
                scan_window(hist, true, inv_tau, false, z1, 0, 0.0, vw, Cd, Md, sh, tid);
                find_mass_cut(vw, T, 0, C_hi, M_hi, sh, tid);
                const int hb = sh.cut_bin;
                kept_C = sh.cut_C; kept_M = sh.cut_M;
                __syncthreads();
                best = race_window(hist, true, hb, z1, c, a.seed, grow, RaceBest{-1.0, 0, 0}, sh, tid);
            }
        }
    }

    }   // two-window code

    // the column inside the winning level
    uint32_t w4[4];
    philox4x32_10(0u, (uint32_t)grow, (uint32_t)(grow >> 32), 4u, (uint32_t)a.seed, (uint32_t)(a.seed >> 32), w4);
    const uint64_t k23 = (uint64_t)(w4[0] >> 9);
    int tok = 0;
    if (best.q >= 0.0) {
        const int pos = (int)(((2u * k23 + 1u) * (uint64_t)best.n) >> 24);
        tok = best.n <= kListCap ? locate_listed(rowp, V, best.bits, pos, sh, tid)
                                 : locate_column(rowp, V, best.bits, pos, sh, tid);
        if (tok < 0 || tok >= V) tok = 0;             // only reachable with non-finite input
    }
    if (tid == 0) {
        a.token_out[row] = tok;
        if (a.kept_out) a.kept_out[row] = kept_C;
        if (a.logp_out)
            a.logp_out[row] = best.q >= 0.0
                ? (float)((bf16_value(best.bits) - z1) * inv_tau - log(kept_M))
                : __builtin_nanf("");
    }
}

}  // namespace

hipError_t launch_sample_restricted(const void* logits, int64_t rows, int64_t V, int64_t row_stride,
                                    const float* tau_rows, float tau_scalar, int32_t top_k, float top_p,
                                    uint64_t seed, uint64_t row_base, int32_t* token_out,
                                    float* logp_out, int32_t* kept_out, hipStream_t stream)
{
    if (rows == 0) return hipSuccess;
    RestrictedArgs a;
    a.logits = static_cast<const uint16_t*>(logits);
    a.rows = rows; a.V = V; a.row_stride = row_stride;
    a.tau_rows = tau_rows; a.tau_scalar = tau_scalar;
    a.top_k = top_k; a.top_p = top_p;
    a.seed = seed; a.row_base = row_base;
    a.token_out = token_out; a.logp_out = logp_out; a.kept_out = kept_out;
    hipLaunchKernelGGL(sample_restricted_kernel, dim3((unsigned)rows), dim3(kRThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace e3
