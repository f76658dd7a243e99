// Vocabulary pass for gfx950: one coalesced HBM read of a [rows, V] logit matrix
// that yields, per row, the entropy of softmax(z / tau), the log-probability of a
// sampled or given token and (rollout side) a two-level Gumbel-max sample.
//
// Paper: arXiv 2505.18573.  Softmax with temperature and the Shannon entropy are
// Appendix A's; the entropy is evaluated through the appendix's decomposition
// H = beta * sum_i p_i Delta_i + ln Z(beta), which in running-reference form is
// H = ln S - W/S with S = sum exp(a_i - ref), W = sum (a_i - ref) exp(a_i - ref).
// The paper samples rollouts "at temperature tau" (Section 5.1) without describing
// a sampler; the two-level Gumbel-max used here is specified in include/e3.h.
//
// Work decomposition (wave = 64 lanes):
//   * a row is cut into super-tiles of 8192 columns; one wave streams a whole
//     super-tile as 16 sweeps of 64 lanes x 8 columns (16 bytes of bf16 per lane),
//     so every load instruction of a wave covers 1 KiB of contiguous memory;
//   * the 16 chunks one lane sees inside a super-tile are exactly one sampler tile,
//     so per-tile sums never leave the lane's registers;
//   * each wave keeps one integer-valued log2 reference `rc` shared by its lanes
//     (SGPR); it only moves when a sweep holds a new maximum, and moving it rescales
//     by an exact power of two;
//   * lanes accumulate in fp32, lane->wave->row merges run in fp64;
//   * waves of a workgroup take super-tiles round-robin and meet once in LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "vocab_pass.h"

namespace e3 {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Tunables (overridable at compile time for experiments).
#ifndef E3_AHEAD_BF16
#define E3_AHEAD_BF16 16     // 16 sweeps x 1 KiB = 16 KiB per wave in flight
#endif
#ifndef E3_AHEAD_F32
#define E3_AHEAD_F32 8       // 8 sweeps x 2 KiB
#endif
#ifndef E3_NT_LOADS
#define E3_NT_LOADS 1        // stream the logits with non-temporal loads
#endif

constexpr int kChunk = 8;                       // columns per lane per sweep
constexpr int kLanes = 64;                      // lanes = tiles per super-tile
constexpr int kDepth = 16;                      // sweeps per super-tile
constexpr int kSweepCols = kChunk * kLanes;     // 512
constexpr int kSuperCols = kSweepCols * kDepth; // 8192
constexpr double kLog2e = 1.4426950408889634074;
constexpr double kLn2 = 0.69314718055994530942;

// ---------------------------------------------------------------------------
// Wave-level reductions on DPP (data-parallel primitives): butterflies inside a
// row of 16 lanes (two quad permutes, half-row mirror, row mirror), then the
// row_bcast15 / row_bcast31 steps that leave the total in lane 63.
// ---------------------------------------------------------------------------
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // row_half_mirror
constexpr int kDppMirror = 0x140;     // row_mirror
constexpr int kDppBcast15 = 0x142;    // lane 15 of each row -> next row   (row mask 0xA)
constexpr int kDppBcast31 = 0x143;    // lane 31 -> rows 2 and 3           (row mask 0xC)

template <int kCtrl, int kRowMask = 0xF>
__device__ __forceinline__ int dpp_i(int old, int v)
{
    return __builtin_amdgcn_update_dpp(old, v, kCtrl, kRowMask, 0xF, false);
}
template <int kCtrl, int kRowMask = 0xF>
__device__ __forceinline__ float dpp_f(float old, float v)
{
    return __int_as_float(dpp_i<kCtrl, kRowMask>(__float_as_int(old), __float_as_int(v)));
}
template <int kCtrl, int kRowMask = 0xF>
__device__ __forceinline__ double dpp_d(double old, double v)
{
    const int lo = dpp_i<kCtrl, kRowMask>(__double2loint(old), __double2loint(v));
    const int hi = dpp_i<kCtrl, kRowMask>(__double2hiint(old), __double2hiint(v));
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ float last_lane(float v)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Maximum over the wave, returned wave-uniform.  One DPP-modified v_max_f32 per
// step (asm, so that no operand canonicalisation is added); the s_nop covers the
// VALU-write -> DPP-read hazard of this ISA family.
__device__ __forceinline__ float wave_max(float v)
{
    asm("s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(v));
    return last_lane(v);
}

// Sum over the wave in fp64, returned wave-uniform.
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_d<kDppXor1>(0.0, v);
    v += dpp_d<kDppXor2>(0.0, v);
    v += dpp_d<kDppHalfMirror>(0.0, v);
    v += dpp_d<kDppMirror>(0.0, v);
    v += dpp_d<kDppBcast15, 0xA>(0.0, v);
    v += dpp_d<kDppBcast31, 0xC>(0.0, v);
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ float uniform_f(float v)
{
    return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(v)));
}

// Three-input maximum as one VALU instruction.  Written as asm because the
// compiler would first canonicalise every operand that came out of integer
// unpacking (one extra instruction per logit).
__device__ __forceinline__ float fmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Candidate of a Gumbel-max race: larger weight wins, equal weights go to the
// lower index.
struct Cand { float q; int idx; };

__device__ __forceinline__ Cand better(Cand a, Cand b)
{
    bool take_b = (b.q > a.q) || (b.q == a.q && b.idx < a.idx);
    return take_b ? b : a;
}

template <int kCtrl, int kRowMask = 0xF>
__device__ __forceinline__ Cand best_step(Cand c)
{
    Cand o;
    o.q = dpp_f<kCtrl, kRowMask>(c.q, c.q);       // rows masked off see themselves: a no-op
    o.idx = dpp_i<kCtrl, kRowMask>(c.idx, c.idx);
    return better(c, o);
}

// Best candidate of the wave, returned wave-uniform.
__device__ __forceinline__ Cand wave_best(Cand c)
{
    c = best_step<kDppXor1>(c);
    c = best_step<kDppXor2>(c);
    c = best_step<kDppHalfMirror>(c);
    c = best_step<kDppMirror>(c);
    c = best_step<kDppBcast15, 0xA>(c);
    c = best_step<kDppBcast31, 0xC>(c);
    Cand r;
    r.q = last_lane(c.q);
    r.idx = __builtin_amdgcn_readlane(c.idx, 63);
    return r;
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11) and the exponential variate -ln(u).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4])
{
    constexpr uint32_t MA = 0xD2511F53u, MB = 0xCD9E8D57u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t ha = __umulhi(MA, c0), la = MA * c0;
        uint32_t hb = __umulhi(MB, c2), lb = MB * c2;
        uint32_t n0 = hb ^ c1 ^ k0;
        uint32_t n2 = ha ^ c3 ^ k1;
        c0 = n0; c1 = lb; c2 = n2; c3 = la;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// E = -ln(u), u = ((word >> 9) + 1/2) 2^-23.  u and d = 1 - u are exact in fp32.
// Close to u = 1 the logarithm is taken from the series -ln(1-d) = sum d^k / k,
// which keeps full relative accuracy where log(u) itself would cancel.
__device__ __forceinline__ float exp_variate(uint32_t word)
{
    float k = (float)(word >> 9);
    float u = fmaf(k, 0x1p-23f, 0x1p-24f);
    float d = 1.0f - u;
    float series = d * fmaf(d, fmaf(d, fmaf(d, fmaf(d, fmaf(d, fmaf(d, 1.0f / 7.0f, 1.0f / 6.0f),
                   0.2f), 0.25f), 1.0f / 3.0f), 0.5f), 1.0f);
    float direct = -logf(u);
    return d < 0.0625f ? series : direct;
}

__device__ __forceinline__ u32x4 stream_load(const u32x4* p)
{
#if E3_NT_LOADS
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

// ---------------------------------------------------------------------------
// chunk loaders: 8 consecutive columns of one lane as fp32
// ---------------------------------------------------------------------------
struct ChunkBf16 {
    u32x4 v;
    static constexpr int kElemBytes = 2;
    static constexpr int kAhead = E3_AHEAD_BF16;   // sweeps kept in flight per wave
    __device__ __forceinline__ void load(const char* row, int64_t col)
    {
        v = stream_load(reinterpret_cast<const u32x4*>(row + col * 2));
    }
    __device__ __forceinline__ void unpack(float z[8]) const
    {
        z[0] = __uint_as_float(v.x << 16); z[1] = __uint_as_float(v.x & 0xFFFF0000u);
        z[2] = __uint_as_float(v.y << 16); z[3] = __uint_as_float(v.y & 0xFFFF0000u);
        z[4] = __uint_as_float(v.z << 16); z[5] = __uint_as_float(v.z & 0xFFFF0000u);
        z[6] = __uint_as_float(v.w << 16); z[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
    static __device__ __forceinline__ float load_one(const char* row, int64_t col)
    {
        return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(row)[col] << 16);
    }
};

struct ChunkF32 {
    u32x4 a, b;
    static constexpr int kElemBytes = 4;
    static constexpr int kAhead = E3_AHEAD_F32;    // sweeps kept in flight per wave
    __device__ __forceinline__ void load(const char* row, int64_t col)
    {
        const u32x4* p = reinterpret_cast<const u32x4*>(row + col * 4);
        a = stream_load(p);
        b = stream_load(p + 1);
    }
    __device__ __forceinline__ void unpack(float z[8]) const
    {
        z[0] = __uint_as_float(a.x); z[1] = __uint_as_float(a.y);
        z[2] = __uint_as_float(a.z); z[3] = __uint_as_float(a.w);
        z[4] = __uint_as_float(b.x); z[5] = __uint_as_float(b.y);
        z[6] = __uint_as_float(b.z); z[7] = __uint_as_float(b.w);
    }
    static __device__ __forceinline__ float load_one(const char* row, int64_t col)
    {
        return reinterpret_cast<const float*>(row)[col];
    }
};

// ---------------------------------------------------------------------------
// Running state of one wave.  rc, top, dom_lane and dom_open are wave-uniform.
// All sums are in base-2 units relative to rc:  t = z*c - rc,  e = 2^t.
//
// The largest logit the wave has met so far (`top`, the one that last moved the
// reference) is kept OUT of the fp32 sums and carried as a scalar.  On a peaked row
// that term is ~1 while all others together may be 1e-4 or less; inside an fp32
// accumulator it would swallow their low bits (absolute error ~1e-7), kept apart the
// remaining sums stay accurate relative to themselves and the row merge can form
// ln S and the entropy from log1p(rest / dominant) without cancellation.
// ---------------------------------------------------------------------------
struct LaneState {
    float rc;          // shared reference = ceil(top * c), -inf before the first element
    float top;         // the excluded maximum (a stored logit value), -inf before the first
    int dom_lane;      // lane whose chunk held `top`
    bool dom_open;     // `top` belongs to that lane's tile that is still open
    float S, W;        // finished tiles:   sum e,  sum t*e
    float sT0, sT1;    // current tile (two chains for instruction-level parallelism)
    float wT0, wT1;
    Cand best;         // best tile so far: q = tile mass / E_tile, idx = tile id
};

// A logit slot that must not count (past the end of the row, or the excluded
// maximum) is filled with this value: t = z*c - rc stays finite, 2^t flushes to
// exactly 0 and t*0 = 0, so it drops out of every sum without any masking.
// Real logits are required to be far above it (|z| < 1e30).
constexpr float kAbsent = -1.0e30f;

// A sweep holds a logit above the wave's reference.  Move the reference to
// ceil(new top * c): the shift d is a non-negative integer, so scaling by 2^-d is
// exact.  The previous top becomes an ordinary term of the lane that held it; the new
// one is struck from its chunk.
__device__ __forceinline__ void new_maximum(LaneState& s, float z[8], float chunk_max, float c,
                                            int lane)
{
    const float top = wave_max(chunk_max);
    float new_rc = ceilf(top * c);
    if (fmaf(top, c, -new_rc) > 0.0f) new_rc += 1.0f;   // product rounded down onto an integer
    new_rc = uniform_f(new_rc);
    if (s.rc > -INFINITY) {
        const float d = new_rc - s.rc;
        const float f = __builtin_amdgcn_exp2f(-d);           // exact: d is an integer
        s.W = fmaf(-d, s.S, s.W) * f;       s.S *= f;
        s.wT0 = fmaf(-d, s.sT0, s.wT0) * f; s.sT0 *= f;
        s.wT1 = fmaf(-d, s.sT1, s.wT1) * f; s.sT1 *= f;
        s.best.q *= f;
        const float t_old = fmaf(s.top, c, -new_rc);
        const float e_old = __builtin_amdgcn_exp2f(t_old);
        if (lane == s.dom_lane) {
            if (s.dom_open) { s.sT0 += e_old; s.wT0 = fmaf(t_old, e_old, s.wT0); }
            else            { s.S += e_old;   s.W = fmaf(t_old, e_old, s.W); }
        }
    }
    s.rc = new_rc;
    s.top = top;
    const unsigned long long holders = __ballot(chunk_max == top);
    s.dom_lane = __builtin_amdgcn_readfirstlane((int)__builtin_ctzll(holders | (1ull << 63)));
    s.dom_open = true;
    bool done = lane != s.dom_lane;
#pragma unroll
    for (int j = 0; j < 8; ++j) {                               // strikes the lowest such j only
        const bool hit = !done && z[j] == top;
        z[j] = hit ? kAbsent : z[j];
        done = done || hit;
    }
}

// Accumulate one chunk of 8 logits (absent slots already hold kAbsent).
__device__ __forceinline__ void accumulate_chunk(LaneState& s, float z[8], float c, int lane)
{
    const float cm = fmax3(fmax3(z[0], z[1], z[2]), fmax3(z[3], z[4], z[5]), fmax3(z[6], z[7], z[7]));
    // t_max > 0: the reference no longer covers this sweep (always so while rc = -inf)
    const float tmax = fmaf(cm, c, -s.rc);
    if (__builtin_expect(__any(tmax > 0.0f), 0)) new_maximum(s, z, cm, c, lane);
    const float nrc = -s.rc;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float t = fmaf(z[j], c, nrc);
        const float e = __builtin_amdgcn_exp2f(t);
        if (j & 1) { s.sT1 += e; s.wT1 = fmaf(t, e, s.wT1); }
        else       { s.sT0 += e; s.wT0 = fmaf(t, e, s.wT0); }
    }
}

// Close the lane's current tile: fold it into the row sums and, when sampling, enter
// it into the level-1 race with weight mass / E.  The tile that holds the excluded
// maximum counts it in its mass.
template <bool kSample>
__device__ __forceinline__ void close_tile(LaneState& s, int tile, float inv_e, bool nonempty,
                                           float c, int lane)
{
    const float sT = s.sT0 + s.sT1;
    const float wT = s.wT0 + s.wT1;
    s.S += sT;
    s.W += wT;
    if (kSample && nonempty) {
        float mass = sT;
        if (s.dom_open && lane == s.dom_lane)
            mass += __builtin_amdgcn_exp2f(fmaf(s.top, c, -s.rc));
        Cand cand{mass * inv_e, tile};
        if (cand.q > s.best.q) s.best = cand;
    }
    s.dom_open = false;
    s.sT0 = s.sT1 = s.wT0 = s.wT1 = 0.0f;
}

// What one wave hands to the workgroup merge.
struct WavePartial {
    double S, W;       // sums over the wave's columns except `top`, relative to rc
    float rc, top;
    float q;           // the wave's best level-1 weight, relative to rc
    int tile;
};

template <typename Chunk, int kWaves, bool kSample>
__global__ __launch_bounds__(kWaves * 64)
void vocab_pass_kernel(VocabPassArgs a)
{
    __shared__ WavePartial partial[kWaves];
    __shared__ float tile_inv_e[kSample ? kWaves : 1][4][kLanes];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row = blockIdx.x;
    const int64_t V = a.V;
    const char* rowp = static_cast<const char*>(a.logits)
                     + row * a.row_stride * (int64_t)Chunk::kElemBytes;

    const int nst = (int)((V + kSuperCols - 1) / kSuperCols);   // super-tiles in a row
    const int nfull = (int)(V / kSuperCols);                    // of which complete

    // Rolling prefetch: kAhead sweeps stay requested ahead of the one being consumed
    // (16 KiB per wave in flight); sweep i lives in buf[i % kAhead].  The first
    // requests leave before anything else is looked at.
    constexpr int kAhead = Chunk::kAhead;
    Chunk buf[kAhead];
    const int64_t lane_col = (int64_t)lane * kChunk;
    if (wave < nfull) {
#pragma unroll
        for (int i = 0; i < kAhead; ++i)
            buf[i].load(rowp, (int64_t)wave * kSuperCols + i * kSweepCols + lane_col);
    }

    const float tau = a.tau_rows ? a.tau_rows[row] : a.tau_scalar;
    const float c = (float)(kLog2e / (double)tau);
    const uint64_t grow = a.row_base + (uint64_t)row;
    const uint32_t row_lo = (uint32_t)grow, row_hi = (uint32_t)(grow >> 32);
    const uint32_t seed_lo = (uint32_t)a.seed, seed_hi = (uint32_t)(a.seed >> 32);

    // Training side: the target's logit is requested now and used in the epilogue.
    // (Read from a clamped column without a branch, so that nothing waits on it here.)
    int64_t tgt = -1;
    float z_tgt = 0.0f;
    if (!kSample) {
        if (a.target_ids != nullptr) tgt = a.target_ids[row];
        const int64_t safe = tgt < 0 ? 0 : (tgt >= V ? V - 1 : tgt);
        z_tgt = Chunk::load_one(rowp, safe);
    }

    LaneState s;
    s.rc = -INFINITY;
    s.top = -INFINITY;
    s.dom_lane = 0;
    s.dom_open = false;
    s.S = s.W = s.sT0 = s.sT1 = s.wT0 = s.wT1 = 0.0f;
    s.best = Cand{-1.0f, 0};

    // Tile noise for four of this wave's super-tiles at a time (the k-th to (k+3)-th
    // it visits): lane l draws the Philox block that serves tiles 4j..4j+3 (j = l % 16)
    // of the (k + l / 16)-th one.  The table is private to the wave; LDS operations of
    // one wave complete in order, so a wave-level fence is all the ordering it needs.
    auto refill_tile_noise = [&](int st_first) {
        const int st_n = st_first + (lane >> 4) * kWaves;
        uint32_t w[4];
        philox4x32_10((uint32_t)(st_n * 16 + (lane & 15)), row_lo, row_hi, 1u, seed_lo, seed_hi, w);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            tile_inv_e[kSample ? wave : 0][lane >> 4][(lane & 15) * 4 + j] = 1.0f / exp_variate(w[j]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    // Complete super-tiles: wave, wave + kWaves, ...  While another complete one
    // follows, the sweep kAhead further on is requested as soon as a sweep has been
    // unpacked, unconditionally, so the loads in flight never drain; the last complete
    // super-tile runs the same body without reaching into a successor.
    int k = 0;
    int st = wave;
    auto run_super_tile = [&](auto prefetch) {
        float inv_e = 0.0f;
        if (kSample) {
            if ((k & 3) == 0) refill_tile_noise(st);
            inv_e = tile_inv_e[wave][k & 3][lane];
        }
        const int64_t this_base = (int64_t)st * kSuperCols + lane_col;
        const int64_t next_base = (int64_t)(st + kWaves) * kSuperCols + lane_col;
#pragma unroll
        for (int i = 0; i < kDepth; ++i) {
            float z[8];
            buf[i % kAhead].unpack(z);
            if (i + kAhead < kDepth)
                buf[i % kAhead].load(rowp, this_base + (i + kAhead) * kSweepCols);
            else if (decltype(prefetch)::value)
                buf[i % kAhead].load(rowp, next_base + (i + kAhead - kDepth) * kSweepCols);
            accumulate_chunk(s, z, c, lane);
        }
        close_tile<kSample>(s, st * kLanes + lane, inv_e, true, c, lane);
        st += kWaves;
        ++k;
    };
    while (st + kWaves < nfull) run_super_tile(std::true_type{});
    if (st < nfull) run_super_tile(std::false_type{});

    // The one incomplete super-tile of the row, if any, belongs to the wave whose turn
    // it is; k already counts the super-tiles that wave has done.  Its sweeps are taken
    // in two halves of 8: guarded loads of a half are all issued before the first is used.
    if (nst > nfull && wave == nfull % kWaves) {
        st = nfull;
        float inv_e = 0.0f;
        if (kSample) {
            if ((k & 3) == 0) refill_tile_noise(st);
            inv_e = tile_inv_e[wave][k & 3][lane];
        }
        const int64_t base = (int64_t)st * kSuperCols + lane_col;
        bool any_valid = false;
#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            const int64_t hbase = base + (int64_t)half * (kDepth / 2) * kSweepCols;
            if (hbase - lane_col >= V) break;                    // uniform: nothing left
            Chunk rb[kDepth / 2];
#pragma unroll
            for (int i = 0; i < kDepth / 2; ++i)
                if (hbase + i * kSweepCols + kChunk <= V) rb[i].load(rowp, hbase + i * kSweepCols);
#pragma unroll
            for (int i = 0; i < kDepth / 2; ++i) {
                const int64_t col = hbase + i * kSweepCols;
                float z[8];
                bool valid = false;
                if (col + kChunk <= V) {
                    rb[i].unpack(z);
                    valid = true;
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        z[j] = kAbsent;
                        if (col + j < V) { z[j] = Chunk::load_one(rowp, col + j); valid = true; }
                    }
                }
                any_valid |= valid;
                if (__any(valid)) accumulate_chunk(s, z, c, lane);
            }
        }
        close_tile<kSample>(s, st * kLanes + lane, inv_e, any_valid, c, lane);
    }

    // lane -> wave, in fp64 (all lanes of a wave share rc, so plain sums)
    const double Sw = wave_sum((double)s.S);
    const double Ww = wave_sum((double)s.W);
    const Cand wb = wave_best(s.best);

    // Rollout side: each wave requests the columns of its own best tile right away
    // (32 lanes x 4 consecutive columns), so that whichever wave wins the row already
    // holds them when the winner is known.
    float cz[4] = {kAbsent, kAbsent, kAbsent, kAbsent};
    int64_t ccol0 = 0;
    if (kSample) {
        const int cst = wb.idx / kLanes, cslot = wb.idx % kLanes;
        ccol0 = (int64_t)cst * kSuperCols + (int64_t)(lane >> 1) * kSweepCols
              + (int64_t)cslot * kChunk + (lane & 1) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (lane < 32 && ccol0 + j < V) cz[j] = Chunk::load_one(rowp, ccol0 + j);
    }

    if (lane == 0) {
        partial[wave].S = Sw;
        partial[wave].W = Ww;
        partial[wave].rc = s.rc;
        partial[wave].top = s.top;
        partial[wave].q = wb.q;
        partial[wave].tile = wb.idx;
    }
    __syncthreads();

    // wave -> row.  R is the common reference, `peak` the largest logit of the row.
    // The wave that owns the winning tile finishes the row (wave 0 on the training side).
    float R = -INFINITY, peak = -INFINITY;
    int peak_wave = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        R = fmaxf(R, partial[w].rc);
        if (partial[w].top > peak) { peak = partial[w].top; peak_wave = w; }
    }
    int owner = 0;
    if (kSample) {
        double best_q = -1.0;
        int best_tile = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float rcw = partial[w].rc;
            if (!(rcw > -INFINITY)) continue;                 // wave had no columns
            const double d = (double)R - (double)rcw;         // integer >= 0
            const double q = ldexp((double)partial[w].q, d > 4000.0 ? -4000 : -(int)d);
            if (q > best_q || (q == best_q && partial[w].tile < best_tile)) {
                best_q = q;
                best_tile = partial[w].tile;
                owner = w;
            }
        }
    }
    if (wave != owner) return;

    // Every lane of the finishing wave repeats the same scalar merge.  Each other
    // wave's excluded maximum joins the rest as an ordinary term.
    const double cd = (double)c;
    double S_rest = 0.0, W_rest = 0.0;   // relative to R, peak excluded
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const float rcw = partial[w].rc;
        if (!(rcw > -INFINITY)) continue;
        const double d = (double)R - (double)rcw;
        const int sh = d > 4000.0 ? -4000 : -(int)d;
        S_rest += ldexp(partial[w].S, sh);
        W_rest += ldexp(partial[w].W - d * partial[w].S, sh);
        if (w != peak_wave) {
            const double tw = (double)partial[w].top * cd - (double)R;
            const double ew = (double)exp2f((float)tw);
            S_rest += ew;
            W_rest += tw * ew;
        }
    }
    // With e_p = 2^{t_p} the peak's term, x = S_rest / e_p and y = W_rest / e_p:
    //   ln S = t_p ln2 + log1p(x),   H = ln S - ln2 W / S = log1p(x) + ln2 (t_p x - y) / (1 + x),
    // every piece of which is O(x) when the row is peaked.  t_p lies in (-1, 0].
    const double t_p = (double)peak * cd - (double)R;
    const double inv_ep = (double)exp2f((float)-t_p);
    const double x = S_rest * inv_ep, y = W_rest * inv_ep;
    const double l1p = (double)log1pf((float)x);
    const double H = l1p + kLn2 * (t_p * x - y) / (1.0 + x);

    int64_t tok;
    float z_tok;
    if (kSample) {
        // Level 2: Gumbel-max inside the winning tile (already in cz), in race form:
        // maximise 2^{(z - zmax) c} / E_col.
        const float zmax = wave_max(fmaxf(fmaxf(cz[0], cz[1]), fmaxf(cz[2], cz[3])));
        uint32_t w[4];
        philox4x32_10((uint32_t)(ccol0 >> 2), row_lo, row_hi, 2u, seed_lo, seed_hi, w);
        Cand cb{-1.0f, 0x7FFFFFFF};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool ok = lane < 32 && ccol0 + j < V;
            const float q = __builtin_amdgcn_exp2f((cz[j] - zmax) * c) / exp_variate(w[j]);
            cb = better(cb, Cand{ok ? q : -1.0f, ok ? (int)(ccol0 + j) : 0x7FFFFFFF});
        }
        cb = wave_best(cb);
        tok = cb.idx;
        if (tok < 0 || tok >= V) tok = 0;                 // only reachable with non-finite input
        float mine = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (ccol0 + j == tok) mine = cz[j];
        z_tok = wave_max(mine);
        if (lane == 0) a.token_out[row] = (int32_t)tok;
    } else {
        tok = tgt;
        z_tok = z_tgt;
    }

    if (lane == 0) {
        if (a.entropy_out) a.entropy_out[row] = (float)H;
        if (a.logp_out) {
            float lp = __builtin_nanf("");
            if (tok >= 0 && tok < V)   // ln p = (a_tok - a_peak) - log1p(x)
                lp = (float)(((double)z_tok - (double)peak) * cd * kLn2 - l1p);
            a.logp_out[row] = lp;
        }
    }
}

// ---------------------------------------------------------------------------
// Batch entropy sum for the scheduler's H_t (mean entropy of the current step,
// Eq. 4): one workgroup, fp64, fixed summation order.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024)
void entropy_reduce_kernel(const float* __restrict__ entropy, const uint8_t* __restrict__ mask,
                           int64_t rows, double* sum_out, int64_t* count_out)
{
    __shared__ double ssum[16];
    __shared__ long long scnt[16];
    double acc = 0.0;
    long long cnt = 0;
    for (int64_t r = threadIdx.x; r < rows; r += 1024) {
        if (!mask || mask[r]) { acc += (double)entropy[r]; ++cnt; }
    }
    acc = wave_sum(acc);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { ssum[wave] = acc; scnt[wave] = cnt; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        long long n = 0;
        for (int w = 0; w < 16; ++w) { t += ssum[w]; n += scnt[w]; }
        if (sum_out) *sum_out = t;
        if (count_out) *count_out = (int64_t)n;
    }
}

// ---------------------------------------------------------------------------
// host-side launchers
// ---------------------------------------------------------------------------
template <typename Chunk, bool kSample, int kWaves>
static hipError_t launch_rows(const VocabPassArgs& a, hipStream_t stream)
{
    dim3 grid((unsigned)a.rows), block(kWaves * 64);
    hipLaunchKernelGGL((vocab_pass_kernel<Chunk, kWaves, kSample>), grid, block, 0, stream, a);
    return hipGetLastError();
}

// Waves per row.  A row of the 151,936-column vocabulary has 19 super-tiles; four
// waves share them 5/5/5/4.
static int pick_waves(const VocabPassArgs& a)
{
#ifdef E3_FORCE_WAVES
    return E3_FORCE_WAVES;
#else
    (void)a;
    return 4;
#endif
}

template <typename Chunk, bool kSample>
static hipError_t launch_for(const VocabPassArgs& a, hipStream_t stream)
{
    switch (pick_waves(a)) {
        case 16: return launch_rows<Chunk, kSample, 16>(a, stream);
        case 8: return launch_rows<Chunk, kSample, 8>(a, stream);
        default: return launch_rows<Chunk, kSample, 4>(a, stream);
    }
}

hipError_t launch_vocab_pass(const VocabPassArgs& a, bool is_bf16, bool sample, hipStream_t stream)
{
    if (a.rows == 0) return hipSuccess;
    if (is_bf16)
        return sample ? launch_for<ChunkBf16, true>(a, stream)
                      : launch_for<ChunkBf16, false>(a, stream);
    return sample ? launch_for<ChunkF32, true>(a, stream)
                  : launch_for<ChunkF32, false>(a, stream);
}

hipError_t launch_entropy_reduce(const float* entropy, const uint8_t* mask, int64_t rows,
                                 double* sum_out, int64_t* count_out, hipStream_t stream)
{
    hipLaunchKernelGGL(entropy_reduce_kernel, dim3(1), dim3(1024), 0, stream,
                       entropy, mask, rows, sum_out, count_out);
    return hipGetLastError();
}

}  // namespace e3
