// Restricted (top-k, optionally followed by top-p) sampling for small k, bf16 and fp32
// rows, for gfx950.
//
// Paper: arXiv 2505.18573 samples its rollouts unrestricted at temperature tau (Section
// 5.1); the truncations are the library's own definition, stated in include/e3.h on value
// LEVELS (the columns that store one bit pattern).  restricted.hip implements it for bf16
// rows through a histogram of all 65,536 patterns; that costs one LDS atomic per column and
// cannot hold the 2^32 patterns of fp32.  For top_k <= 256 the kept set is tiny, and this
// file finds it by selection instead:
//   1. one streaming read of the row leaves the maximum of every chunk of columns in LDS
//      (plain vector maxima: about two instructions per column, no atomics) and every
//      thread's own maximum in a register;
//   2. theta, a value that at least k of the thread maxima reach, is a lower bound of the k-th
//      largest column (k different threads hold a column at or above it), and a tight one:
//      only the few chunks whose maximum reaches theta can hold kept columns;
//   3. the columns at or above theta are read again from those chunks and listed in LDS; an
//      exact radix select over them gives kappa, the value of the cut level, with the number
//      of columns above it (fewer than k) and on it;
//   4. the columns above kappa are listed, sorted by (value, column), grouped into levels
//      with their fp64 masses, cut by top-p, raced and the winning level's pos-th column
//      taken, exactly as the definition says; the cut level takes part with its count.
// Every count is exact and every mass fp64, as in restricted.hip; a row with enormous
// plateaus of equal values is slow (its chunks all qualify) but takes the same path.
// Steps 3 (from the radix select on) and 4 exist twice: workgroup-wide, with a barrier after
// every short phase, and - for a list of at most 256 candidates and top_k <= 64, the usual
// case - inside one wave with the kept columns one per lane (finish_in_one_wave below).
#include "vocab_common.h"
#include "vocab_pass.h"

namespace e3 {
namespace {

// Threads per row.  Measured on MI355X, 512 rows x 151,936, top-k 50, workgroup-wide steps
// throughout: 512 threads with up to 128 registers each (two workgroups per compute unit,
// nothing spilled) 49.9 us for bf16 rows and 80 us for fp32 rows; 1024 threads held to 64
// registers (the same two workgroups per compute unit; a dozen spilled, whose reloads queue
// behind the streaming) 61.7 - 67 us and 82 - 112 us.
#ifndef E3_SEL_THREADS
#define E3_SEL_THREADS 512
#endif
constexpr int kSThreads = E3_SEL_THREADS;
constexpr int kSWaves = kSThreads / 64;
constexpr int kSBatch = 4096 / kSThreads;          // 16-byte requests a thread keeps in flight: 64 KiB per workgroup
constexpr int kSMaxK = 256;             // top_k served here; the gt-list holds at most kSMaxK - 1 columns
constexpr int kSEqCap = 64;             // columns of the cut level listed for a direct pick
constexpr int kSListCap = 2048;         // candidates (columns at or above theta) listed in LDS
constexpr uint32_t kKeyPosZero = 0x80000000u, kKeyNegZero = 0x7FFFFFFFu;

// Monotone map of a binary32 pattern to an unsigned key (value order, -0 just below +0);
// patterns that are not finite numbers get key 0, below every level.
__device__ __forceinline__ uint32_t key_of_f32(uint32_t bits)
{
    if ((bits & 0x7F800000u) == 0x7F800000u) return 0u;
    return (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
}
__device__ __forceinline__ uint32_t f32_of_key(uint32_t key)
{
    return (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;
}

// Element access for the two logit types.  A vector is 16 bytes.  Keys are 32-bit in
// registers; bf16 rows store their chunk maxima as the upper 16 bits (the lower 16 of a bf16
// value's key are all ones or all zeros and can be rebuilt).
struct SelBf16 {
    typedef uint16_t Stored;
    static constexpr int kElems = 8;
    static constexpr int kChunksPerThreadMax = 20 * 1024 / kSThreads;   // 40 KiB of chunk maxima
    static constexpr int kKeyBits = 16;              // significant key bits, from the top
    static __device__ __forceinline__ uint32_t elem_bits(const u32x4& v, int j)   // as binary32
    {
        const uint32_t w = j < 2 ? v.x : j < 4 ? v.y : j < 6 ? v.z : v.w;
        return (j & 1) ? (w & 0xFFFF0000u) : (w << 16);
    }
    static __device__ __forceinline__ Stored pack(uint32_t key) { return (Stored)(key >> 16); }
    // the largest key with these upper bits: never below the key that was packed
    static __device__ __forceinline__ uint32_t unpack_upper(Stored s) { return ((uint32_t)s << 16) | 0xFFFFu; }
    static __device__ __forceinline__ uint32_t pattern_of_bits(uint32_t bits) { return bits >> 16; }
    static __device__ __forceinline__ float vec_max(const u32x4& v)
    {
        return fmax3(fmax3(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16)),
                     fmax3(__uint_as_float(v.y & 0xFFFF0000u), __uint_as_float(v.z << 16), __uint_as_float(v.z & 0xFFFF0000u)),
                     fmaxf(__uint_as_float(v.w << 16), __uint_as_float(v.w & 0xFFFF0000u)));
    }
};
struct SelF32 {
    typedef uint32_t Stored;
    static constexpr int kElems = 4;
    static constexpr int kChunksPerThreadMax = 10 * 1024 / kSThreads;   // 40 KiB of chunk maxima
    static constexpr int kKeyBits = 32;
    static __device__ __forceinline__ uint32_t elem_bits(const u32x4& v, int j)
    {
        return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w;
    }
    static __device__ __forceinline__ Stored pack(uint32_t key) { return key; }
    static __device__ __forceinline__ uint32_t unpack_upper(Stored s) { return s; }
    static __device__ __forceinline__ uint32_t pattern_of_bits(uint32_t bits) { return bits; }
    static __device__ __forceinline__ float vec_max(const u32x4& v)
    {
        return fmax3(fmax3(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z)),
                     __uint_as_float(v.w), __uint_as_float(v.w));
    }
};

struct alignas(16) SelShared {
    uint32_t hist[256];
    uint32_t prefix, k_rem, n_eq_last;      // radix select state
    uint32_t n_total;                        // candidates seen by the first pass
    int gt_n, eq_n, list_n;                  // list fills
    int pad_;                                // keeps the arrays below on 16-byte boundaries
    int rank[kSMaxK];
    uint32_t gt_key[kSMaxK];                 // unsorted, then sorted by (key desc, col asc)
    int32_t gt_col[kSMaxK];
    uint32_t st_key[kSMaxK];
    int32_t st_col[kSMaxK];
    double st_M[kSMaxK];                     // inclusive prefix mass in sorted order
    int32_t eq_col[kSEqCap];
    int cut_index;                           // last kept entry of the sorted list (-1: none), or kSMaxK: cut level kept
    float wave_q[kSWaves];
    int wave_lvl[kSWaves];
    int wave_hits[kSWaves];
    int token;
    uint32_t tmax_wave[kSWaves];
};

static_assert(offsetof(SelShared, gt_key) % 16 == 0 && offsetof(SelShared, gt_col) % 16 == 0, "read four at a time");

// One 8-bit pass of a radix select for the k-th largest: every thread has added its keys
// that match `prefix` above `shift + 8` to hist; wave 0 finds the digit that holds rank k_rem.
__device__ __forceinline__ void select_digit(SelShared& sh, int tid)
{
    if (tid < 64) {
        // lane l owns bins 255 - 4l .. 252 - 4l (descending)
        uint32_t c[4], sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { c[j] = sh.hist[255 - 4 * tid - j]; sum += c[j]; }
        uint32_t inc = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(inc, d, 64);
            if (tid >= d) inc += o;
        }
        uint32_t before = inc - sum;                       // counts in higher bins
        const uint32_t k = sh.k_rem;
        if (before < k && k <= inc) {                       // exactly one lane
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (before < k && k <= before + c[j]) {
                    sh.prefix = (sh.prefix << 8) | (uint32_t)(255 - 4 * tid - j);
                    sh.k_rem = k - before;
                    sh.n_eq_last = c[j];
                    before = 0xFFFFFFFFu;                   // done
                } else if (before != 0xFFFFFFFFu) {
                    before += c[j];
                }
            }
        }
    }
}

// Inclusive prefix sum over the lanes of a wave: four shifts inside each row of sixteen lanes,
// then lane 15 of a row into the next row and lane 31 into the upper half (lanes a shift does
// not reach read zero).
__device__ __forceinline__ int wave_prefix_sum(int v)
{
    v += dpp_i<0x111>(0, v);               // row_shr:1
    v += dpp_i<0x112>(0, v);               // row_shr:2
    v += dpp_i<0x114>(0, v);               // row_shr:4
    v += dpp_i<0x118>(0, v);               // row_shr:8
    v += dpp_i<kDppBcast15, 0xA>(0, v);
    v += dpp_i<kDppBcast31, 0xC>(0, v);
    return v;
}

struct SelArgs {
    const void* logits;
    int64_t rows, V, row_stride;
    const float* tau_rows;
    float tau_scalar;
    int32_t top_k;
    float top_p;
    uint64_t seed, row_base;
    int32_t* token_out;
    float* logp_out;
    int32_t* kept_out;
    int group;            // vectors per chunk
    int chunks;           // chunks per thread
};

// ---------------------------------------------------------------------------
// The rest of a row in one wave, for a short candidate list (at most kSoloList entries in
// LDS) and a small count cut (top_k <= kSoloK, so fewer than 64 columns stand above the cut
// level: one per lane, and lane 63 is free for the cut level itself).  Same steps and same
// arithmetic as the workgroup-wide code in the kernel below; what changes is where the
// data sit: the list is held in registers (four entries per lane), kappa is found bit by bit
// with ballots, the columns above it then live one per lane, are ranked against each other
// through lane broadcasts, and masses, cuts, race and pick are wave scans, ballots and lane
// reads.  No workgroup barrier is involved (the other waves
// have left), and what goes through LDS is ordered by the wave's own program order.
// ---------------------------------------------------------------------------
constexpr int kSoloList = 256;
constexpr int kSoloK = 64;

__device__ __forceinline__ double read_lane_f64(double v, int src_lane)
{
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xFFFFFFFFll), src_lane);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), src_lane);
    return __longlong_as_double(((long long)hi << 32) | (long long)(uint32_t)lo);
}

template <typename T>
__device__ __forceinline__ void finish_in_one_wave(const SelArgs& a, SelShared& sh, const uint32_t* lkey,
                                                   const int32_t* lcol, int n_list, int k_req, int64_t row,
                                                   uint64_t grow, double inv_tau, float c, int lane)
{
    auto lds_order = []() {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    const unsigned long long below = (1ull << lane) - 1ull;        // lanes before mine

    // the list in registers: lane l holds entries l, l + 64, ... (key 0 = none: below every real key)
    constexpr int kPerLane = kSoloList / 64;
    uint32_t lk[kPerLane];
    int32_t lc[kPerLane];
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
        const int e = lane + 64 * j;
        lk[j] = e < n_list ? lkey[e] : 0u;
        lc[j] = e < n_list ? lcol[e] : 0;
    }
    // kappa, the k-th largest listed key, bit by bit from the top: the largest value that at
    // least k keys reach (one ballot per register and bit; the keys' low bits follow the sign
    // when only the upper kKeyBits are significant)
    const int k_eff = n_list < k_req ? n_list : k_req;              // fewer than k finite columns: all of them
    uint32_t kappa = 0u;
    for (int b = 31; b >= 32 - T::kKeyBits; --b) {
        const uint32_t cand = kappa | (1u << b);
        int reach = 0;
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) reach += __popcll(__ballot(lk[j] >= cand));
        if (reach >= k_eff) kappa = cand;
    }
    if (T::kKeyBits < 32 && (kappa & 0x80000000u) == 0u) kappa |= 0xFFFFFFFFu >> T::kKeyBits;

    // the columns above kappa, one per lane in list order; those on kappa's level into their list
    uint32_t key_i = 0u;
    int32_t col_i = 0;
    int n = 0, n_cut = 0;                                          // columns above kappa (fewer than k), columns on its level
    {
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            const bool gt = lk[j] > kappa;
            const unsigned long long gm = __ballot(gt);
            if (gt) {
                const int slot = n + __popcll(gm & below);
                sh.gt_key[slot] = lk[j];
                sh.gt_col[slot] = lc[j];
            }
            n += __popcll(gm);
            const bool eq = lk[j] == kappa;
            const unsigned long long em = __ballot(eq);
            if (eq) {
                const int slot = n_cut + __popcll(em & below);
                if (slot < kSEqCap) sh.eq_col[slot] = lc[j];
            }
            n_cut += __popcll(em);
        }
        lds_order();
        if (lane < n) { key_i = sh.gt_key[lane]; col_i = sh.gt_col[lane]; }
    }
    // rank by (value descending, column ascending): each lane counts the lanes ahead of it; one
    // 64-bit comparison per pair on (key, inverted column)
    const uint64_t order_i = ((uint64_t)key_i << 32) | (uint32_t)~col_i;
    int rank = 0;
    for (int e = 0; e < n; ++e) {
        const uint32_t ok = (uint32_t)__builtin_amdgcn_readlane((int)key_i, e);
        const uint32_t oc = (uint32_t)__builtin_amdgcn_readlane(~col_i, e);
        rank += (((uint64_t)ok << 32) | oc) > order_i;
    }
    if (lane < n) { sh.st_key[rank] = key_i; sh.st_col[rank] = col_i; }
    lds_order();
    const bool have = lane < n;
    const uint32_t skey = have ? sh.st_key[lane] : 0u;             // lane = rank from here on
    const int32_t scol = have ? sh.st_col[lane] : 0;

    // masses in rank order (fp64), cuts
    const uint32_t key1 = n > 0 ? (uint32_t)__builtin_amdgcn_readlane((int)skey, 0) : kappa;   // the row's highest level
    const double z1 = (double)__uint_as_float(f32_of_key(key1));
    const double z_cut = (double)__uint_as_float(f32_of_key(kappa));
    const double w = have ? exp(((double)__uint_as_float(f32_of_key(skey)) - z1) * inv_tau) : 0.0;
    double M = w;                                                   // inclusive prefix mass
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const double o = __shfl_up(M, d, 64);
        if (lane >= d) M += o;
    }
    const double M_gt = n > 0 ? read_lane_f64(M, n - 1) : 0.0;
    const double w_cut = exp((z_cut - z1) * inv_tau);
    const double M_k = M_gt + (double)n_cut * w_cut;               // mass of the top-k set
    const uint32_t next_key = (uint32_t)__shfl_down((int)skey, 1, 64);
    const uint32_t prev_key = (uint32_t)__shfl_up((int)skey, 1, 64);
    int cut_index = kSMaxK;                                          // default: everything down to the cut level
    if (a.top_p < 1.0f) {
        // top-p on the renormalised top-k set: first level end whose cumulative mass reaches the target
        const double Tm = (double)a.top_p * M_k;
        const bool level_end = have && (lane == n - 1 || next_key != skey);
        const unsigned long long reach = __ballot(level_end && M >= Tm);
        if (reach != 0ull) cut_index = (int)__builtin_ctzll(reach);
    }
    const bool cut_level_kept = cut_index == kSMaxK;
    const int kept_sorted = cut_level_kept ? n : cut_index + 1;    // sorted entries kept
    const int kept_C = cut_level_kept ? n + n_cut : kept_sorted;
    const double kept_M = cut_level_kept ? M_k : read_lane_f64(M, cut_index);

    // race of the kept levels: a level's first lane scores it, lane 63 scores the cut level
    const bool level_start = have && (lane == 0 || prev_key != skey);
    const unsigned long long starts = __ballot(level_start);
    const unsigned long long later = lane < 63 ? starts >> (lane + 1) : 0ull;
    const int cnt = (later != 0ull ? lane + 1 + (int)__builtin_ctzll(later) : n) - lane;    // columns of my level
    const float z1f = __uint_as_float(f32_of_key(key1));
    const bool for_cut = lane == 63 && cut_level_kept;
    float my_q = -1.0f;
    int my_lvl = 0x7FFFFFFF;                                       // sorted index of the level's first entry; kSMaxK = cut level
    if ((level_start && lane < kept_sorted) || for_cut) {
        const uint32_t bits = f32_of_key(for_cut ? kappa : skey);
        const uint32_t pat = T::pattern_of_bits(bits);
        uint32_t w4[4];
        philox4x32_10(pat >> 2, (uint32_t)grow, (uint32_t)(grow >> 32), 3u,
                      (uint32_t)a.seed, (uint32_t)(a.seed >> 32), w4);
        const int sel = pat & 3;
        const uint32_t word = sel == 0 ? w4[0] : sel == 1 ? w4[1] : sel == 2 ? w4[2] : w4[3];
        my_q = (float)(for_cut ? n_cut : cnt) * __builtin_amdgcn_exp2f((__uint_as_float(bits) - z1f) * c)
             * inv_exp_variate(word);
        my_lvl = for_cut ? kSMaxK : lane;
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const float oq = __shfl_xor(my_q, d, 64);
        const int ol = __shfl_xor(my_lvl, d, 64);
        if (oq > my_q || (oq == my_q && ol < my_lvl)) { my_q = oq; my_lvl = ol; }   // ties: the higher level
    }
    const float best_q = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, my_q)));
    const int best_lvl = __builtin_amdgcn_readfirstlane(my_lvl);

    // the column inside the winning level
    uint32_t w4[4];
    philox4x32_10(0u, (uint32_t)grow, (uint32_t)(grow >> 32), 4u, (uint32_t)a.seed, (uint32_t)(a.seed >> 32), w4);
    const uint64_t k23 = (uint64_t)(w4[0] >> 9);
    int tok = 0;
    uint32_t tok_key = key1;
    if (best_q >= 0.0f && best_lvl < kSMaxK) {
        const int level_cnt = __builtin_amdgcn_readlane(cnt, best_lvl);
        const int pos = (int)(((2u * k23 + 1u) * (uint64_t)level_cnt) >> 24);
        tok = __builtin_amdgcn_readlane(scol, best_lvl + pos);     // a level's lanes are in column order
        tok_key = (uint32_t)__builtin_amdgcn_readlane((int)skey, best_lvl);
    } else if (best_q >= 0.0f) {
        const int pos = (int)(((2u * k23 + 1u) * (uint64_t)n_cut) >> 24);
        tok_key = kappa;
        if (n_cut <= kSEqCap) {
            // the pos-th smallest of the level's listed columns
            const int32_t mc = lane < n_cut ? sh.eq_col[lane] : 0x7FFFFFFF;
            int before = 0;
            for (int e = 0; e < n_cut; ++e) before += __builtin_amdgcn_readlane(mc, e) < mc;
            const unsigned long long hit = __ballot(lane < n_cut && before == pos);
            tok = __builtin_amdgcn_readlane(mc, (int)__builtin_ctzll(hit | (1ull << 63)));
        } else {
            // a longer level inside the list: rank its columns against each other from LDS
            for (int e0 = 0; e0 < n_list; e0 += 64) {
                const int e = e0 + lane;
                const bool mine = e < n_list && lkey[e] == kappa;
                const int32_t mc = e < n_list ? lcol[e] : 0;
                int before = 0;
                if (mine)
                    for (int f = 0; f < n_list; ++f) before += lkey[f] == kappa && lcol[f] < mc;
                const unsigned long long hit = __ballot(mine && before == pos);
                if (hit != 0ull) tok = __builtin_amdgcn_readlane(mc, (int)__builtin_ctzll(hit));
            }
        }
    }
    if (lane == 0) {
        if (tok < 0 || tok >= a.V) tok = 0;
        a.token_out[row] = tok;
        if (a.kept_out) a.kept_out[row] = kept_C;
        if (a.logp_out)
            a.logp_out[row] = best_q >= 0.0f
                ? (float)(((double)__uint_as_float(f32_of_key(tok_key)) - z1) * inv_tau - log(kept_M))
                : __builtin_nanf("");
    }
}

// Two workgroups per compute unit: kSWaves / 2 waves per SIMD, which bounds the registers a
// wave may take (512 / that many vector registers, 800 / that many scalar ones).
template <typename T>
__global__ __launch_bounds__(kSThreads) __attribute__((amdgpu_waves_per_eu(kSWaves / 2, kSWaves / 2)))
void sample_select_kernel(SelArgs a)
{
    extern __shared__ __align__(16) unsigned char dyn[];
    typename T::Stored* cmax = reinterpret_cast<typename T::Stored*>(dyn);
    __shared__ SelShared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int64_t V = a.V;
    const int esz = 16 / T::kElems;
    const char* rowp = static_cast<const char*>(a.logits) + row * a.row_stride * esz;
    const u32x4* rv = reinterpret_cast<const u32x4*>(rowp);
    const int64_t nvec = (V + T::kElems - 1) / T::kElems;     // the last one may reach past V (inside the row pitch)
    const int G = a.group, CPT = a.chunks;
    const float tau = a.tau_rows ? a.tau_rows[row] : a.tau_scalar;
    const double inv_tau = 1.0 / (double)tau;
    const float c = kLog2eF / tau;
    const uint64_t grow = a.row_base + (uint64_t)row;

    // ---- 1. chunk maxima ------------------------------------------------------------------
    // chunk j of thread t = vectors t + kSThreads (j G + g), g < G.  Maxima are taken as floats
    // (NaN operands drop out of v_max3); +inf is dealt with below; a maximum of zero is
    // recorded as +0, whichever zero it was.
    auto vec_key_max = [&](int64_t v, const u32x4& x) -> uint32_t {
        float m = T::vec_max(x);
        if (v == nvec - 1 && nvec * T::kElems != V) {           // columns past V do not count
            m = -INFINITY;
            for (int j = 0; j < T::kElems; ++j)
                if (v * T::kElems + j < V) m = fmaxf(m, __uint_as_float(T::elem_bits(x, j)));
        }
        uint32_t key = m == 0.0f ? kKeyPosZero : key_of_f32(__float_as_uint(m));
        if (m == INFINITY) {                                      // skip the non-finite ones by hand
            key = 0u;
            for (int j = 0; j < T::kElems; ++j)
                if (v * T::kElems + j < V) {
                    const uint32_t kj = key_of_f32(T::elem_bits(x, j));
                    key = kj > key ? kj : key;
                }
        }
        return key;
    };
    // Vector slots s = j G + g of this thread, kSBatch requests in flight at a time.
    uint32_t tmax = 0u;
    {
        const int nslots = CPT * G;
        uint32_t m = 0u;                                          // maximum of the chunk being filled
        for (int s0 = 0; s0 < nslots; s0 += kSBatch) {
            u32x4 x[kSBatch];
            int64_t vv[kSBatch];
#pragma unroll
            for (int u = 0; u < kSBatch; ++u) {
                vv[u] = (int64_t)tid + (int64_t)kSThreads * (s0 + u);
                x[u] = (s0 + u < nslots && vv[u] < nvec) ? rv[vv[u]] : u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int u = 0; u < kSBatch; ++u) {
                const int sl = s0 + u;
                if (sl < nslots) {
                    if (vv[u] < nvec) { const uint32_t k1 = vec_key_max(vv[u], x[u]); m = k1 > m ? k1 : m; }
                    if ((sl + 1) % G == 0) {                      // last vector of chunk sl / G
                        cmax[(size_t)(sl / G) * kSThreads + tid] = T::pack(m);
                        tmax = m > tmax ? m : tmax;
                        m = 0u;
                    }
                }
            }
        }
    }

    // ---- 2. theta: the k-th largest thread maximum ---------------------------------------------
    const unsigned long long have_w = __ballot(tmax != 0u);
    if (lane == 0) sh.wave_hits[wave] = __popcll(have_w);
    if (tid == 0) { sh.gt_n = 0; sh.eq_n = 0; sh.token = 0; }
    __syncthreads();
    int n_threads_with = 0;
    for (int w = 0; w < kSWaves; ++w) n_threads_with += sh.wave_hits[w];
    __syncthreads();
    if (n_threads_with == 0) {                                    // no finite logit in the row
        if (tid == 0) {
            a.token_out[row] = 0;
            if (a.kept_out) a.kept_out[row] = 0;
            if (a.logp_out) a.logp_out[row] = __builtin_nanf("");
        }
        return;
    }
    // Each wave takes the m-th largest of its lanes' maxima, m = ceil(k / kSWaves), bit by bit
    // from the top with one ballot per bit (the largest value that at least m lanes reach; the
    // bits below the significant ones stay zero, which only lowers the bound); the smallest of
    // the waves' results has kSWaves m >= k threads at or above it.  No atomics, one barrier.
    // (The exact k-th largest of the thread maxima would be a little tighter; it costs two to
    // four histogram passes with their barriers.)
    const int k_req = a.top_k < kSMaxK ? a.top_k : kSMaxK;
    uint32_t theta;
    {
        const int m_th = (k_req + kSWaves - 1) / kSWaves;
        uint32_t wm = 0u;
        for (int b = 31; b >= 32 - T::kKeyBits; --b) {
            const uint32_t cand = wm | (1u << b);
            if ((int)__popcll(__ballot(tmax >= cand)) >= m_th) wm = cand;
        }
        if (lane == 0) sh.tmax_wave[wave] = wm;
        __syncthreads();
        theta = 0xFFFFFFFFu;
        for (int w = 0; w < kSWaves; ++w) theta = sh.tmax_wave[w] < theta ? sh.tmax_wave[w] : theta;
        if (theta == 0u) theta = 1u;                                // a wave with fewer than m finite maxima: every finite value
        // a zero maximum was recorded as +0 whichever zero it was: let -0 in as well
        if (theta == kKeyPosZero) theta = kKeyNegZero;
    }

    // ---- 3. the candidates: every finite column whose key reaches theta ----------------------------
    // They sit in the chunks whose maximum reaches theta.  Usually there are a few hundred: they
    // are read once more and listed in LDS (key, column), and everything below works on the list.
    // A row with huge plateaus of equal values overflows the list; it is then read from memory
    // in every pass instead (slow, same results).
    uint32_t* lkey = reinterpret_cast<uint32_t*>(dyn + (size_t)CPT * kSThreads * sizeof(typename T::Stored));
    int32_t* lcol = reinterpret_cast<int32_t*>(lkey + kSListCap);
    auto stream_candidates = [&](auto&& f) {
        for (int j = 0; j < CPT; ++j) {
            if (T::unpack_upper(cmax[(size_t)j * kSThreads + tid]) < theta) continue;
            for (int g = 0; g < G; ++g) {
                const int64_t v = (int64_t)tid + (int64_t)kSThreads * ((int64_t)j * G + g);
                if (v >= nvec) break;
                const u32x4 x = rv[v];
#pragma unroll
                for (int e = 0; e < T::kElems; ++e) {
                    const int64_t col = v * T::kElems + e;
                    const uint32_t key = key_of_f32(T::elem_bits(x, e));
                    if (col < V && key >= theta) f(key, (int32_t)col);
                }
            }
        }
    };
    // one slot per true flag, one LDS atomic per wave instruction
    auto wave_slot = [&](bool flag, int* counter) -> int {
        const unsigned long long m = __ballot(flag);
        if (m == 0ull) return -1;
        int base = 0;
        const int leader = (int)__builtin_ctzll(m);
        if (lane == leader) base = atomicAdd(counter, __popcll(m));
        base = __shfl(base, leader, 64);
        return base + __popcll(m & ((1ull << lane) - 1ull));
    };
    if (tid == 0) sh.list_n = 0;
    __syncthreads();
    {
        // The thread's qualifying chunks as a bit mask; their vectors are then walked four at a
        // time with fixed register slots (a register array indexed by a running count would
        // live in scratch memory, and each of its accesses would queue behind the other rows'
        // streaming).  All lanes of a wave take part in every round: the slot reservation is
        // a wave-wide operation.
        static_assert(T::kChunksPerThreadMax <= 64, "one mask bit per chunk");
        uint64_t qmask = 0u;
        for (int j = 0; j < CPT; ++j)
            qmask |= (uint64_t)(T::unpack_upper(cmax[(size_t)j * kSThreads + tid]) >= theta) << j;
        int j = qmask != 0u ? __builtin_ctzll(qmask) : -1, g = 0;
        while (__any(j >= 0)) {
            int64_t vq[4];
            bool on[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                vq[u] = (int64_t)tid + (int64_t)kSThreads * ((int64_t)(j < 0 ? 0 : j) * G + g);
                on[u] = j >= 0 && vq[u] < nvec;
                if (j >= 0 && (++g == G || !on[u])) {              // next qualifying chunk
                    g = 0;
                    qmask &= qmask - 1u;
                    j = qmask != 0u ? __builtin_ctzll(qmask) : -1;
                }
            }
            u32x4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) x[u] = on[u] ? rv[vq[u]] : u32x4{0u, 0u, 0u, 0u};
            // count my candidates, reserve a run of slots for the wave, write mine in order
            uint32_t ok_mask = 0u;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
#pragma unroll
                for (int e = 0; e < T::kElems; ++e) {
                    const int64_t col = vq[u] * T::kElems + e;
                    const uint32_t key = key_of_f32(T::elem_bits(x[u], e));
                    ok_mask |= (uint32_t)(on[u] && col < V && key >= theta) << (u * T::kElems + e);
                }
            }
            const int mine = __popc(ok_mask);
            const int inc = wave_prefix_sum(mine);
            const int wave_total = __builtin_amdgcn_readlane(inc, 63);
            int base = 0;
            if (lane == 63 && wave_total > 0) base = atomicAdd(&sh.list_n, wave_total);
            base = __builtin_amdgcn_readlane(base, 63);
            int slot = base + inc - mine;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
#pragma unroll
                for (int e = 0; e < T::kElems; ++e) {
                    if (ok_mask & (1u << (u * T::kElems + e))) {
                        if (slot < kSListCap) {
                            lkey[slot] = key_of_f32(T::elem_bits(x[u], e));
                            lcol[slot] = (int32_t)(vq[u] * T::kElems + e);
                        }
                        ++slot;
                    }
                }
            }
        }
    }
    __syncthreads();
    const int n_list = sh.list_n;
    const bool listed = n_list <= kSListCap;
    if (n_list <= kSoloList && k_req <= kSoloK) {                  // short list, small k: one wave finishes the row
        if (wave == 0) finish_in_one_wave<T>(a, sh, lkey, lcol, n_list, k_req, row, grow, inv_tau, c, lane);
        return;
    }
    auto for_each_candidate = [&](auto&& f) {
        if (listed) {
            for (int e = tid; e < n_list; e += kSThreads) f(lkey[e], lcol[e]);
        } else {
            stream_candidates(f);
        }
    };

    // ---- 4. kappa: the k-th largest column (exact), by radix select over the candidates ---------
    if (tid == 0) { sh.prefix = 0u; sh.k_rem = 0u; sh.n_total = 0u; }
    uint32_t k_col = (uint32_t)k_req;
    for (int pass = 0; pass < T::kKeyBits / 8; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) sh.hist[tid] = 0u;
        __syncthreads();
        const uint32_t prefix = sh.prefix;
        for_each_candidate([&](uint32_t key, int32_t) {
            if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
        });
        __syncthreads();
        if (pass == 0) {
            // number of candidates; fewer than k finite columns in the row: the cut is the lowest level
            if (tid < 64) {
                uint32_t t = sh.hist[tid] + sh.hist[tid + 64] + sh.hist[tid + 128] + sh.hist[tid + 192];
#pragma unroll
                for (int d = 32; d > 0; d >>= 1) t += __shfl_xor(t, d, 64);
                if (tid == 0) { sh.n_total = t; sh.k_rem = t < k_col ? t : k_col; }
            }
            __syncthreads();
        }
        select_digit(sh, tid);
        __syncthreads();
    }
    const uint32_t kappa = T::kKeyBits == 32 ? sh.prefix
                         : ((sh.prefix << 16) | ((sh.prefix & 0x8000u) ? 0u : 0xFFFFu));   // rebuild a bf16 value's key
    const int n_cut = (int)sh.n_eq_last;                          // columns on the cut level
    const uint32_t k_eff = sh.n_total < k_col ? sh.n_total : k_col;
    const int count_gt = (int)(k_eff - sh.k_rem);                 // columns above it (< k)
    __syncthreads();

    // ---- 5. the columns above kappa, and those on it when they are few -------------------------------
    if (listed) {
        for (int e0 = 0; e0 < n_list; e0 += kSThreads) {          // whole waves: wave_slot is wave-wide
            const int e = e0 + tid;
            const uint32_t key = e < n_list ? lkey[e] : 0u;
            const int32_t col = e < n_list ? lcol[e] : 0;
            const int sg = wave_slot(key > kappa, &sh.gt_n);
            if (key > kappa && sg < kSMaxK) { sh.gt_key[sg] = key; sh.gt_col[sg] = col; }
            const bool eq = key == kappa && n_cut <= kSEqCap;
            const int se = wave_slot(eq, &sh.eq_n);
            if (eq && se < kSEqCap) sh.eq_col[se] = col;
        }
    } else {
        stream_candidates([&](uint32_t key, int32_t col) {
            if (key > kappa) {
                const int slot = atomicAdd(&sh.gt_n, 1);
                if (slot < kSMaxK) { sh.gt_key[slot] = key; sh.gt_col[slot] = col; }
            } else if (key == kappa && n_cut <= kSEqCap) {
                const int slot = atomicAdd(&sh.eq_n, 1);
                if (slot < kSEqCap) sh.eq_col[slot] = col;
            }
        });
    }
    __syncthreads();
    const int n = count_gt;                                        // == sh.gt_n
    // sort by (key descending, column ascending): rank by counting, the n x n comparisons spread
    // over all threads (entry i = tid mod 256 against one part of the others each)
    if (tid < kSMaxK) sh.rank[tid] = 0;
    __syncthreads();
    {
        constexpr int kParts = kSThreads / kSMaxK;
        static_assert(kParts >= 1 && kParts * kSMaxK == kSThreads, "whole parts");
        const int i = tid & (kSMaxK - 1), part = tid / kSMaxK;
        if (i < n) {
            // four entries per LDS read, one 64-bit comparison per pair on (key, inverted column)
            const uint64_t mine = ((uint64_t)sh.gt_key[i] << 32) | (uint32_t)~sh.gt_col[i];
            const int per = ((n + kParts - 1) / kParts + 3) & ~3;
            const int e_begin = part * per;
            const int e_end = e_begin + per < n ? e_begin + per : n;
            int r = 0;
            for (int e = e_begin; e < e_end; e += 4) {
                const uint4 ok = *reinterpret_cast<const uint4*>(&sh.gt_key[e]);
                const int4 oc = *reinterpret_cast<const int4*>(&sh.gt_col[e]);
                r += (((uint64_t)ok.x << 32) | (uint32_t)~oc.x) > mine;
                r += e + 1 < e_end && (((uint64_t)ok.y << 32) | (uint32_t)~oc.y) > mine;
                r += e + 2 < e_end && (((uint64_t)ok.z << 32) | (uint32_t)~oc.z) > mine;
                r += e + 3 < e_end && (((uint64_t)ok.w << 32) | (uint32_t)~oc.w) > mine;
            }
            if (r != 0) atomicAdd(&sh.rank[i], r);
        }
    }
    __syncthreads();
    if (tid < n) {
        const int r = sh.rank[tid];
        sh.st_key[r] = sh.gt_key[tid];
        sh.st_col[r] = sh.gt_col[tid];
    }
    __syncthreads();

    // ---- 6. masses in rank order (fp64), cuts -----------------------------------------------------
    const uint32_t key1 = n > 0 ? sh.st_key[0] : kappa;           // the row's highest level
    const double z1 = (double)__uint_as_float(f32_of_key(key1));
    const double z_cut = (double)__uint_as_float(f32_of_key(kappa));
    if (tid < n) sh.st_M[tid] = exp(((double)__uint_as_float(f32_of_key(sh.st_key[tid])) - z1) * inv_tau);
    __syncthreads();
    if (tid < 64) {
        // wave 0: lane l holds sorted entries 4l .. 4l+3; inclusive prefix sums in rank order
        double w[4], loc = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = 4 * tid + j;
            w[j] = i < n ? sh.st_M[i] : 0.0;
            loc += w[j];
        }
        double inc = loc;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const double o = __shfl_up(inc, d, 64);
            if (tid >= d) inc += o;
        }
        double run = inc - loc;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = 4 * tid + j;
            run += w[j];
            if (i < n) sh.st_M[i] = run;
        }
    }
    __syncthreads();
    const double M_gt = n > 0 ? sh.st_M[n - 1] : 0.0;
    const double w_cut = exp((z_cut - z1) * inv_tau);
    const double M_k = M_gt + (double)n_cut * w_cut;              // mass of the top-k set
    // top-p on the renormalised top-k set: first level end whose cumulative mass reaches T
    if (tid == 0) sh.cut_index = kSMaxK;                           // default: everything down to the cut level
    __syncthreads();
    if (a.top_p < 1.0f) {
        const double Tm = (double)a.top_p * M_k;
        if (tid < n) {
            const bool level_end = tid == n - 1 || sh.st_key[tid + 1] != sh.st_key[tid];
            if (level_end && sh.st_M[tid] >= Tm) atomicMin(&sh.cut_index, tid);
        }
        __syncthreads();
    }
    const int cut_index = sh.cut_index;
    const bool cut_level_kept = cut_index == kSMaxK;
    const int kept_sorted = cut_level_kept ? n : cut_index + 1;    // sorted entries kept
    const int kept_C = cut_level_kept ? n + n_cut : kept_sorted;
    const double kept_M = cut_level_kept ? M_k : sh.st_M[cut_index];

    // ---- 7. race of the kept levels ------------------------------------------------------------------
    // score n_j w_j / E_j, E_j from Philox stream 3 at index = the level's stored pattern; fp32
    // scores as in the unrestricted sampler; ties go to the higher level = lower sorted index.
    const float z1f = __uint_as_float(f32_of_key(key1));
    auto level_score = [&](uint32_t key, int cnt) -> float {
        const uint32_t bits = f32_of_key(key);
        const uint32_t pat = T::pattern_of_bits(bits);
        uint32_t w4[4];
        philox4x32_10(pat >> 2, (uint32_t)grow, (uint32_t)(grow >> 32), 3u,
                      (uint32_t)a.seed, (uint32_t)(a.seed >> 32), w4);
        const int sel = pat & 3;
        const uint32_t word = sel == 0 ? w4[0] : sel == 1 ? w4[1] : sel == 2 ? w4[2] : w4[3];
        return (float)cnt * __builtin_amdgcn_exp2f((__uint_as_float(bits) - z1f) * c) * inv_exp_variate(word);
    };
    float my_q = -1.0f;
    int my_lvl = 0x7FFFFFFF;                                       // sorted index of the level's first entry; kSMaxK = cut level
    if (tid < kept_sorted) {
        const bool level_start = tid == 0 || sh.st_key[tid - 1] != sh.st_key[tid];
        if (level_start) {
            int cnt = 1;
            while (tid + cnt < n && sh.st_key[tid + cnt] == sh.st_key[tid]) ++cnt;
            my_q = level_score(sh.st_key[tid], cnt);
            my_lvl = tid;
        }
    } else if (tid == kSThreads - 1 && cut_level_kept) {
        my_q = level_score(kappa, n_cut);
        my_lvl = kSMaxK;
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const float oq = __shfl_xor(my_q, d, 64);
        const int ol = __shfl_xor(my_lvl, d, 64);
        if (oq > my_q || (oq == my_q && ol < my_lvl)) { my_q = oq; my_lvl = ol; }
    }
    if (lane == 0) { sh.wave_q[wave] = my_q; sh.wave_lvl[wave] = my_lvl; }
    __syncthreads();
    float best_q = -1.0f;
    int best_lvl = 0x7FFFFFFF;
    for (int w = 0; w < kSWaves; ++w) {
        const float q = sh.wave_q[w];
        const int l = sh.wave_lvl[w];
        if (q > best_q || (q == best_q && l < best_lvl)) { best_q = q; best_lvl = l; }
    }

    // ---- 8. the column inside the winning level ---------------------------------------------------------
    uint32_t w4[4];
    philox4x32_10(0u, (uint32_t)grow, (uint32_t)(grow >> 32), 4u, (uint32_t)a.seed, (uint32_t)(a.seed >> 32), w4);
    const uint64_t k23 = (uint64_t)(w4[0] >> 9);
    int tok = 0;
    uint32_t tok_key = key1;
    if (best_q >= 0.0f && best_lvl < kSMaxK) {
        int cnt = 1;
        while (best_lvl + cnt < n && sh.st_key[best_lvl + cnt] == sh.st_key[best_lvl]) ++cnt;
        const int pos = (int)(((2u * k23 + 1u) * (uint64_t)cnt) >> 24);
        tok = sh.st_col[best_lvl + pos];                           // a level's entries are in column order
        tok_key = sh.st_key[best_lvl];
    } else if (best_q >= 0.0f) {
        const int pos = (int)(((2u * k23 + 1u) * (uint64_t)n_cut) >> 24);
        tok_key = kappa;
        if (n_cut <= kSEqCap) {
            // the pos-th smallest of the listed columns
            if (tid < n_cut) {
                const int32_t mc = sh.eq_col[tid];
                int rank = 0;
                for (int e = 0; e < n_cut; ++e) rank += sh.eq_col[e] < mc;
                if (rank == pos) sh.token = mc;
            }
            __syncthreads();
            tok = sh.token;
        } else {
            // a plateau: count the level's columns in column order; waves take contiguous runs of vectors
            const int64_t per_wave = (nvec + kSWaves - 1) / kSWaves;
            const int64_t v_begin = (int64_t)wave * per_wave < nvec ? (int64_t)wave * per_wave : nvec;
            const int64_t v_end = v_begin + per_wave < nvec ? v_begin + per_wave : nvec;
            auto mask_of = [&](int64_t v) -> uint32_t {
                const u32x4 x = rv[v];
                uint32_t m = 0;
#pragma unroll
                for (int e = 0; e < T::kElems; ++e)
                    m |= (uint32_t)(v * T::kElems + e < V && key_of_f32(T::elem_bits(x, e)) == kappa) << e;
                return m;
            };
            int hits = 0;
            for (int64_t v = v_begin + lane; v < v_end; v += 64) hits += __popc(mask_of(v));
#pragma unroll
            for (int d = 32; d > 0; d >>= 1) hits += __shfl_xor(hits, d, 64);
            if (lane == 0) sh.wave_hits[wave] = hits;
            __syncthreads();
            int before = 0;
            for (int w = 0; w < wave; ++w) before += sh.wave_hits[w];
            if (pos >= before && pos < before + hits) {            // uniform per wave: my run holds it
                int rem = pos - before;
                for (int64_t v0 = v_begin; v0 < v_end; v0 += 64) {
                    const int64_t v = v0 + lane;
                    const uint32_t m = v < v_end ? mask_of(v) : 0u;
                    const int cc = __popc(m);
                    int inc = cc;
#pragma unroll
                    for (int d = 1; d < 64; d <<= 1) {
                        const int o = __shfl_up(inc, d, 64);
                        if (lane >= d) inc += o;
                    }
                    const int sweep_total = __shfl(inc, 63, 64);
                    if (rem < sweep_total) {
                        if (rem >= inc - cc && rem < inc) {        // exactly one lane
                            int skip = rem - (inc - cc);
                            uint32_t mm = m;
                            while (skip-- > 0) mm &= mm - 1;       // drop the lowest set bits
                            sh.token = (int)(v * T::kElems + (__ffs(mm) - 1));
                        }
                        break;
                    }
                    rem -= sweep_total;
                }
            }
            __syncthreads();
            tok = sh.token;
        }
    }
    if (tid == 0) {
        if (tok < 0 || tok >= V) tok = 0;
        a.token_out[row] = tok;
        if (a.kept_out) a.kept_out[row] = kept_C;
        if (a.logp_out)
            a.logp_out[row] = best_q >= 0.0f
                ? (float)(((double)__uint_as_float(f32_of_key(tok_key)) - z1) * inv_tau - log(kept_M))
                : __builtin_nanf("");
    }
}

}  // namespace

bool sample_select_serves(int32_t top_k) { return top_k >= 1 && top_k <= kSMaxK; }

hipError_t launch_sample_select(const void* logits, bool is_bf16, int64_t rows, int64_t V, int64_t row_stride,
                                const float* tau_rows, float tau_scalar, int32_t top_k, float top_p,
                                uint64_t seed, uint64_t row_base, int32_t* token_out,
                                float* logp_out, int32_t* kept_out, hipStream_t stream)
{
    if (rows == 0) return hipSuccess;
    SelArgs a;
    a.logits = logits; a.rows = rows; a.V = V; a.row_stride = row_stride;
    a.tau_rows = tau_rows; a.tau_scalar = tau_scalar;
    a.top_k = top_k; a.top_p = top_p;
    a.seed = seed; a.row_base = row_base;
    a.token_out = token_out; a.logp_out = logp_out; a.kept_out = kept_out;
    const int elems = is_bf16 ? SelBf16::kElems : SelF32::kElems;
    const int cpt_max = is_bf16 ? SelBf16::kChunksPerThreadMax : SelF32::kChunksPerThreadMax;
    const int64_t nvec = (V + elems - 1) / elems;
    const int64_t vpt = (nvec + kSThreads - 1) / kSThreads;           // vectors per thread
    a.group = (int)((vpt + cpt_max - 1) / cpt_max);
    if (a.group < 1) a.group = 1;
    a.chunks = (int)((vpt + a.group - 1) / a.group);
    const size_t lds = (size_t)a.chunks * kSThreads * (is_bf16 ? sizeof(SelBf16::Stored) : sizeof(SelF32::Stored))
                     + (size_t)kSListCap * 8;
    if (is_bf16)
        hipLaunchKernelGGL(sample_select_kernel<SelBf16>, dim3((unsigned)rows), dim3(kSThreads), lds, stream, a);
    else
        hipLaunchKernelGGL(sample_select_kernel<SelF32>, dim3((unsigned)rows), dim3(kSThreads), lds, stream, a);
    return hipGetLastError();
}

}  // namespace e3
