// Device-side building blocks shared by the vocabulary-pass kernels (gfx950):
// DPP wave reductions, Philox4x32-10 and the exponential variate, 16-byte chunk
// loaders for bf16 / fp32 logits, and the per-lane running softmax state.
//
// Paper: arXiv 2505.18573, Appendix A (temperature softmax, Shannon entropy and its
// decomposition H = beta * sum_i p_i Delta_i + ln Z(beta)); in running-reference
// form H = ln S - W/S with S = sum exp(a_i - ref), W = sum (a_i - ref) exp(a_i - ref).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace e3 {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Tunables (overridable at compile time for experiments).
#ifndef E3_AHEAD_BF16
#define E3_AHEAD_BF16 4      // 4 sweeps x 1 KiB per wave in flight (must divide the tile depth)
#endif
#ifndef E3_AHEAD_F32
#define E3_AHEAD_F32 4       // 4 sweeps x 2 KiB per wave in flight
#endif
#ifndef E3_NT_LOADS
#define E3_NT_LOADS 1        // stream the logits with non-temporal loads
#endif
#ifndef E3_SPLIT_BELOW_NUM        // small-batch path while row-block workgroups <= CUs * NUM / DEN
#define E3_SPLIT_BELOW_NUM 3
#define E3_SPLIT_BELOW_DEN 8
#endif

constexpr int kChunk = 8;                       // columns per lane per sweep
constexpr int kLanes = 64;                      // lanes = tiles per super-tile
constexpr int kDepth = 8;                       // sweeps per super-tile
constexpr int kSweepCols = kChunk * kLanes;     // 512
constexpr int kSuperCols = kSweepCols * kDepth; // 4096
constexpr double kLog2e = 1.4426950408889634074;
constexpr float kLog2eF = 1.44269504088896340736f;
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

// The same over lanes 0..15 only (one DPP row): four butterfly steps leave the row's maximum
// in each of its lanes; lane 0 is read.  For reductions whose operands live in the first
// sixteen lanes (a row's few partials, the sixteen lanes of the sampler's second level).
__device__ __forceinline__ float row16_max(float v)
{
    asm("s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
}

__device__ __forceinline__ double row16_sum(double v)
{
    v += dpp_d<kDppXor1>(0.0, v);
    v += dpp_d<kDppXor2>(0.0, v);
    v += dpp_d<kDppHalfMirror>(0.0, v);
    v += dpp_d<kDppMirror>(0.0, v);
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 0);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 0);
    return __hiloint2double(hi, lo);
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

// Best candidate among lanes 0..15, returned wave-uniform.
__device__ __forceinline__ Cand row16_best(Cand c)
{
    c = best_step<kDppXor1>(c);
    c = best_step<kDppXor2>(c);
    c = best_step<kDppHalfMirror>(c);
    c = best_step<kDppMirror>(c);
    Cand r;
    r.q = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c.q), 0));
    r.idx = __builtin_amdgcn_readlane(c.idx, 0);
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
        const uint64_t pa = (uint64_t)MA * c0, pb = (uint64_t)MB * c2;   // one v_mad_u64_u32 each
        const uint32_t ha = (uint32_t)(pa >> 32), la = (uint32_t)pa;
        const uint32_t hb = (uint32_t)(pb >> 32), lb = (uint32_t)pb;
        // three-input xor in one instruction (bit-operation table 0x96)
        uint32_t n0 = __builtin_amdgcn_bitop3_b32(hb, c1, k0, 0x96);
        uint32_t n2 = __builtin_amdgcn_bitop3_b32(ha, c3, k1, 0x96);
        c0 = n0; c1 = lb; c2 = n2; c3 = la;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// E = -ln(u), u = ((word >> 9) + 1/2) 2^-23 (exact in fp32), through the hardware log2.
// Measured over all 2^23 values of u on gfx950: relative error at most 1.6e-7, also next to
// u = 1, where a logarithm formed from exponent and mantissa tables could have cancelled (a
// seven-term series in 1 - u is no more accurate there: 1.2e-7).  inv_exp_variate is 1 / E
// through the hardware reciprocal (1 ulp): the sampler's scores carry ~3e-7 relative error
// from these two, far inside the 1e-5 near-tie margin.
__device__ __forceinline__ float exp_variate(uint32_t word)
{
    const float k = (float)(word >> 9);
    const float u = fmaf(k, 0x1p-23f, 0x1p-24f);
    return -0.693147180559945309f * __builtin_amdgcn_logf(u);
}

__device__ __forceinline__ float inv_exp_variate(uint32_t word)
{
    return __builtin_amdgcn_rcpf(exp_variate(word));
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
// chunk loaders: 8 consecutive columns (one eighth of a sampler tile) per lane, as fp32.
//   load / unpack              the lane's own 8 columns starting at `col` (any sweep,
//                              also an incomplete one);
//   load_sweep / unpack_sweep  a complete sweep of 512 columns, read so that every load
//                              instruction of the wave covers 1 KiB of contiguous
//                              memory: `col` = first column of the sweep + sweep_col(lane);
//                              after unpack_sweep the lane holds the 8 columns of tile
//                              lane tile_lane(lane) of that sweep.
// ---------------------------------------------------------------------------
struct ChunkBf16 {
    u32x4 v;
    static constexpr int kElemBytes = 2;
    static constexpr int kAhead = E3_AHEAD_BF16;   // sweeps kept in flight per wave
    __device__ __forceinline__ void load(const char* row, int64_t col)
    {
        v = stream_load(reinterpret_cast<const u32x4*>(row + col * 2));
    }
    static __device__ __forceinline__ int sweep_col(int lane) { return lane * 8; }
    static __device__ __forceinline__ int tile_lane(int lane) { return lane; }
    __device__ __forceinline__ void load_sweep(const char* row, int64_t col) { load(row, col); }
    __device__ __forceinline__ void unpack_sweep(float z[8], int) const { unpack(z); }
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
    // largest of the four logits in the high halves of the loaded words (a value the row holds)
    __device__ __forceinline__ float some_max() const
    {
        return fmax3(fmax3(__uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y & 0xFFFF0000u),
                           __uint_as_float(v.z & 0xFFFF0000u)),
                     __uint_as_float(v.w & 0xFFFF0000u), __uint_as_float(v.w & 0xFFFF0000u));
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
    // A sweep of fp32 is 2 KiB: the first load takes 16 bytes per lane from its first
    // KiB, the second from its second KiB.  Lanes 2k and 2k+1 then hold between them
    // tile lane k (first loads) and tile lane 32+k (second loads); they trade halves,
    // so the even lane ends up with tile lane k and the odd one with 32+k.  (Reading the
    // lane's own 32 bytes instead makes every load instruction span 2 KiB half-used.)
    static __device__ __forceinline__ int sweep_col(int lane) { return lane * 4; }
    static __device__ __forceinline__ int tile_lane(int lane) { return (lane >> 1) + ((lane & 1) << 5); }
    __device__ __forceinline__ void load_sweep(const char* row, int64_t col)
    {
        const u32x4* p = reinterpret_cast<const u32x4*>(row + col * 4);
        a = stream_load(p);
        b = stream_load(p + 64);
    }
    __device__ __forceinline__ void unpack_sweep(float z[8], int lane) const
    {
        const bool odd = (lane & 1) != 0;
        const uint32_t keep[4] = {odd ? b.x : a.x, odd ? b.y : a.y, odd ? b.z : a.z, odd ? b.w : a.w};
        const uint32_t give[4] = {odd ? a.x : b.x, odd ? a.y : b.y, odd ? a.z : b.z, odd ? a.w : b.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // quad_perm [1,0,3,2]: every lane reads its neighbour in the pair
            const uint32_t recv = (uint32_t)__builtin_amdgcn_mov_dpp((int)give[i], 0xB1, 0xF, 0xF, true);
            z[i] = __uint_as_float(keep[i]);
            z[4 + i] = __uint_as_float(recv);
        }
    }
    static __device__ __forceinline__ float load_one(const char* row, int64_t col)
    {
        return reinterpret_cast<const float*>(row)[col];
    }
    // largest of the eight loaded logits
    __device__ __forceinline__ float some_max() const
    {
        const float m0 = fmax3(__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(a.z));
        const float m1 = fmax3(__uint_as_float(a.w), __uint_as_float(b.x), __uint_as_float(b.y));
        return fmax3(m0, m1, fmaxf(__uint_as_float(b.z), __uint_as_float(b.w)));
    }
};

// ---------------------------------------------------------------------------
// Running state of one wave.  rc, top, thr, dom_lane and dom_open are wave-uniform.
// All sums are in base-2 units relative to rc:  t = z*c - rc,  e = 2^t.
//
// The largest logit the wave has met above the row's floor (`top`; every new one moves
// the reference) is kept OUT of the fp32 sums and carried as a scalar.  On a peaked row
// that term is ~1 while all others together may be 1e-4 or less; inside an fp32
// accumulator it would swallow their low bits (absolute error ~1e-7), kept apart the
// remaining sums stay accurate relative to themselves and the row merge can form
// ln S and the entropy from log1p(rest / dominant) without cancellation.  The floor is
// a logit value below the row's maximum (or -inf): whatever stays at or under it cannot be
// the row's dominant term and is summed like any other; the row's maximum itself lies
// above every floor, so the wave that meets it does exclude it.
// ---------------------------------------------------------------------------
struct LaneState {
    float rc;          // shared reference: an integer >= (every logit met so far) * c; -inf = none yet
    float top;         // the excluded maximum (a stored logit value), -inf = none yet
    float thr;         // a sweep whose maximum exceeds this moves the reference: max(top, floor)
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

// The integer reference that covers logits up to `z`: ceil(z * c), one more when the fp32
// product was rounded down onto an integer.
__device__ __forceinline__ float reference_for(float z, float c)
{
    float rc = ceilf(z * c);
    if (fmaf(z, c, -rc) > 0.0f) rc += 1.0f;
    return rc;
}

// A sweep holds a logit above the wave's running maximum (and above the floor, see
// start_row).  Move the reference to ceil(new top * c): the shift d is a non-negative
// integer, so scaling by 2^-d is exact.  The previous top becomes an ordinary term of
// the lane that held it; the new one is struck from its chunk.
__device__ __forceinline__ void new_maximum(LaneState& s, float z[8], float chunk_max, float c,
                                            int lane)
{
    const float top = wave_max(chunk_max);
    const float new_rc = uniform_f(reference_for(top, c));
    if (s.rc > -INFINITY && new_rc != s.rc) {                  // wave-uniform
        const float d = new_rc - s.rc;
        const float f = __builtin_amdgcn_exp2f(-d);           // exact: d is an integer
        s.W = fmaf(-d, s.S, s.W) * f;       s.S *= f;
        s.wT0 = fmaf(-d, s.sT0, s.wT0) * f; s.sT0 *= f;
        s.wT1 = fmaf(-d, s.sT1, s.wT1) * f; s.sT1 *= f;
        s.best.q *= f;
    }
    if (s.top > -INFINITY) {                                   // wave-uniform
        const float t_old = fmaf(s.top, c, -new_rc);
        const float e_old = __builtin_amdgcn_exp2f(t_old);
        if (lane == s.dom_lane) {
            if (s.dom_open) { s.sT0 += e_old; s.wT0 = fmaf(t_old, e_old, s.wT0); }
            else            { s.S += e_old;   s.W = fmaf(t_old, e_old, s.W); }
        }
    }
    s.rc = new_rc;
    s.top = top;
    s.thr = top;
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
    // A logit above everything the wave has excluded so far, and above the row's floor,
    // moves the reference; `top` is the running maximum of the wave's logits above the floor.
    if (__builtin_expect(__any(cm > s.thr), 0)) new_maximum(s, z, cm, c, lane);
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

}  // namespace e3
