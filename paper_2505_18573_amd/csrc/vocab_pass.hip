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
//   * a row is cut into super-tiles of 4096 columns; one wave streams a whole
//     super-tile as 8 sweeps of 64 lanes x 8 columns (16 bytes of bf16 per lane),
//     so every load instruction of a wave covers 1 KiB of contiguous memory, and the
//     8 chunks one lane sees are exactly one sampler tile;
//   * a workgroup of 8 waves owns a few whole rows; the super-tiles of those rows are
//     work items dealt to the waves round-robin (wave w takes items w, w + 8, ...), so
//     which columns a wave sums, and in which order, depends on the shape alone and the
//     results are the same bit for bit in every run; a wave keeps the first sweeps of
//     its next item in flight while it finishes the current one;
//   * a wave accumulates the items it gets from one row in registers (fp32 per lane,
//     one integer-valued log2 reference per wave that moves by exact powers of two)
//     and hands over one partial per row; the wave that delivers a row's last item
//     merges the partials in fp64, runs level 2 of the sampler and writes the outputs
//     while the other waves keep streaming.
#include "advantages.h"
#include "vocab_common.h"
#include "vocab_pass.h"
#include <hip/hip_ext.h>
#include <mutex>

namespace e3 {

// What a wave hands over for one row (also: the row's incomplete super-tile).
struct alignas(16) RowPartial {
    double S, W;       // sums over the wave's columns except `top`, relative to rc
    float rc, top;     // reference and excluded maximum; rc = -inf marks an empty slot
    float q;           // mass / E of the best sampler tile among them, relative to rc
    int tile;          // its tile id
};
static_assert(sizeof(RowPartial) == 32, "layout");

// What a wave tells the others about its first work item before the streaming starts: a
// logit value that the item's row holds (see the floor in start_row).
struct WaveHint { int row; float value; };
constexpr int kMaxWaves = 8;

// LDS layout: WaveHint hints[kMaxWaves] | uint32 done[rpb] (padded to 16 B)
//             | RowPartial parts[rpb][kWaves+1] | float inv_e[rpb][nst][64]   (rollout side only)
__host__ __device__ inline size_t lds_done_bytes(int rpb)
{
    return sizeof(WaveHint) * kMaxWaves + (size_t)((rpb * 4 + 15) / 16 * 16);
}

template <int kWaves>
__host__ __device__ inline size_t lds_bytes(int rpb, int nst, bool sample)
{
    return lds_done_bytes(rpb) + sizeof(RowPartial) * (size_t)rpb * (kWaves + 1)
         + (sample ? (size_t)rpb * nst * kLanes * sizeof(float) : 0);
}

// Row epilogue, run by one wave once all of the row's partials are written: merge the
// partials (one per lane, nparts <= 64), level 2 of the sampler or the target gather,
// outputs.  kFew: the partials sit in the first sixteen lanes (a row-block workgroup hands
// over at most nine), so every reduction over them is four DPP steps inside one row of lanes
// instead of six across the wave; level 2 always works on sixteen lanes.  This wave's work
// is a chain of dependent instructions that nothing overlaps once the row is the last of the
// launch, hence the care to keep it short.
template <typename Chunk, bool kSample, bool kFew>
__device__ __forceinline__ void finish_row(const VocabPassArgs& a, int64_t row,
                                           const RowPartial* parts, int nparts, int lane)
{
    const int64_t V = a.V;
    const char* rowp = static_cast<const char*>(a.logits)
                     + row * a.row_stride * (int64_t)Chunk::kElemBytes;
    // training side: ask for the target's logit first, use it last
    int64_t tgt = -1;
    float z_tgt = 0.0f;
    if (!kSample) {
        if (a.target_ids != nullptr) tgt = a.target_ids[row];
        const int64_t safe = tgt < 0 ? 0 : (tgt >= V ? V - 1 : tgt);
        z_tgt = Chunk::load_one(rowp, safe);
    }
    const float tau = a.tau_rows ? a.tau_rows[row] : a.tau_scalar;
    const float c = kLog2eF / tau;

    RowPartial p;
    p.S = 0.0; p.W = 0.0; p.rc = -INFINITY; p.top = -INFINITY; p.q = -1.0f; p.tile = 0;
    if (lane < nparts) p = parts[lane];

    // R is the common reference, `peak` the largest logit of the row; the partial
    // that holds it is the lowest lane with that top, every other excluded maximum
    // joins the rest as an ordinary term.
    const float R = kFew ? row16_max(p.rc) : wave_max(p.rc);
    const float peak = kFew ? row16_max(p.top) : wave_max(p.top);
    const unsigned long long holders = __ballot(p.top == peak);
    const int peak_lane = (int)__builtin_ctzll(holders | (1ull << 63));
    const bool live = p.rc > -INFINITY;
    const double cd = (double)c;
    const double d = live ? (double)R - (double)p.rc : 0.0;       // integer >= 0
    const int sh = d > 4000.0 ? -4000 : -(int)d;

    // Rollout side, level 1 across partials first (weights brought to the common
    // reference by exact scaling), so that the columns of the winning tile are
    // requested before the fp64 merge below and arrive while it runs.
    float cz[4] = {kAbsent, kAbsent, kAbsent, kAbsent};
    float inv_e2[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    int64_t col0 = 0;
    if (kSample) {
        const Cand mine{live ? ldexpf(p.q, sh) : -1.0f, p.tile};
        const Cand win = kFew ? row16_best(mine) : wave_best(mine);
        const int wst = win.idx / kLanes, wslot = win.idx % kLanes;
        // 2 * kDepth lanes x 4 consecutive columns cover the tile
        col0 = (int64_t)wst * kSuperCols + (int64_t)(lane >> 1) * kSweepCols
             + (int64_t)wslot * kChunk + (lane & 1) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (lane < 2 * kDepth && col0 + j < V) cz[j] = Chunk::load_one(rowp, col0 + j);
        const uint64_t grow = a.row_base + (uint64_t)row;
        philox4x32_10((uint32_t)(col0 >> 2), (uint32_t)grow, (uint32_t)(grow >> 32), 2u,
                      (uint32_t)a.seed, (uint32_t)(a.seed >> 32), w);
#pragma unroll
        for (int j = 0; j < 4; ++j) inv_e2[j] = inv_exp_variate(w[j]);   // while the columns arrive
    }

    // Row sums in fp64.
    double S_l = 0.0, W_l = 0.0;
    if (live) {
        S_l = ldexp(p.S, sh);
        W_l = ldexp(p.W - d * p.S, sh);
        if (lane != peak_lane && p.top > -INFINITY) {      // a wave may have excluded nothing
            const double tw = (double)p.top * cd - (double)R;
            const double ew = (double)exp2f((float)tw);
            S_l += ew;
            W_l += tw * ew;
        }
    }
    const double S_rest = kFew ? row16_sum(S_l) : wave_sum(S_l);
    const double W_rest = kFew ? row16_sum(W_l) : wave_sum(W_l);
    // With e_p = 2^{t_p} the peak's term, x = S_rest / e_p and y = W_rest / e_p:
    //   ln S = t_p ln2 + log1p(x),   H = ln S - ln2 W / S = log1p(x) + ln2 (t_p x - y) / (1 + x),
    // every piece of which is O(x) when the row is peaked.  t_p lies in (-1, 0].
    const double t_p = (double)peak * cd - (double)R;
    const double inv_ep = (double)exp2f((float)-t_p);
    const double x = S_rest * inv_ep, y = W_rest * inv_ep;
    const double l1p = (double)log1pf((float)x);
    const double H = l1p + kLn2 * (t_p * x - y) / (1.0 + x);

    if (lane == 0) {
        if (a.entropy_out) a.entropy_out[row] = (float)H;
        if (a.gap_out) {
            // Appendix A's Delta measured on this row: the probability-weighted mean of
            // z_peak - z_i over all other tokens = tau ln2 (t_p - W_rest / S_rest)
            a.gap_out[row] = S_rest > 0.0 ? (float)((double)tau * kLn2 * (t_p - W_rest / S_rest))
                                          : __builtin_nanf("");
        }
    }
    if (kSample) {
        // Level 2: Gumbel-max inside the winning tile, in race form: maximise
        // 2^{(z - z_peak) c} / E_col.  The row's peak serves as the reference: the winning
        // tile's largest column lies within 2^-34 of it (a tile further down cannot make up
        // the difference with its noise, whose range is 2^-24 .. 17), far from underflow.
        Cand cb{-1.0f, 0x7FFFFFFF};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool ok = lane < 2 * kDepth && col0 + j < V;
            const float q = __builtin_amdgcn_exp2f((cz[j] - peak) * c) * inv_e2[j];
            cb = better(cb, Cand{ok ? q : -1.0f, ok ? (int)(col0 + j) : 0x7FFFFFFF});
        }
        cb = row16_best(cb);
        int64_t tok = cb.idx;
        if (tok < 0 || tok >= V) tok = 0;                 // only reachable with non-finite input
        if (lane == 0) a.token_out[row] = (int32_t)tok;
        // the lane that holds the token's column writes its log-probability:
        //   ln p = (a_tok - a_peak) - log1p(x)
        if (a.logp_out) {
            const bool holder = lane < 2 * kDepth && cb.idx >= col0 && cb.idx < col0 + 4;
            if (holder) {
                const int j = (int)(cb.idx - col0);
                const float z_tok = j == 0 ? cz[0] : j == 1 ? cz[1] : j == 2 ? cz[2] : cz[3];
                a.logp_out[row] = (float)(((double)z_tok - (double)peak) * cd * kLn2 - l1p);
            }
            // no column won the race (non-finite logits): the row's outputs are NaN
            if (__ballot(holder) == 0 && lane == 0) a.logp_out[row] = __builtin_nanf("");
        }
    } else if (lane == 0 && a.logp_out) {
        float lp = __builtin_nanf("");
        if (tgt >= 0 && tgt < V)
            lp = (float)(((double)z_tgt - (double)peak) * cd * kLn2 - l1p);
        a.logp_out[row] = lp;
    }
}

// Empty state for a row.  `floor` is a logit value known to be below (or -inf: nothing known
// about) the row's maximum: logits up to the floor are ordinary terms of the sums even when
// they exceed everything this wave has met, and only a logit above it becomes the wave's
// excluded maximum.  The row's largest logit lies above every floor, so the wave that meets it
// excludes it, which is all the row merge needs (it keeps the one dominant term of a peaked
// row out of the fp32 sums); what the floor saves is the reference moves for the many running
// maxima a wave would otherwise meet on its way.
__device__ __forceinline__ void start_row(LaneState& s, float floor, float c)
{
    s.top = -INFINITY; s.dom_lane = 0; s.dom_open = false;
    s.thr = floor;
    s.rc = floor > -INFINITY ? reference_for(floor, c) : -INFINITY;
    s.S = s.W = s.sT0 = s.sT1 = s.wT0 = s.wT1 = 0.0f;
    s.best = Cand{-1.0f, 0};
}

// A row's incomplete last super-tile: sweeps in two halves, the guarded loads of a
// half all issued before the first is used; columns past V count as absent.  Returns
// whether this lane's tile holds any column.
template <typename Chunk>
__device__ __forceinline__ bool stream_ragged(LaneState& s, const char* rowp, int64_t cbase,
                                              int64_t lane_col, int64_t V, float c, int lane)
{
    bool any_valid = false;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const int64_t hbase = cbase + (int64_t)half * (kDepth / 2) * kSweepCols;
        if (hbase - lane_col >= V) break;            // uniform: nothing left
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
    return any_valid;
}

template <typename Chunk, bool kSample, int kWaves, int kAhead>
__global__ __launch_bounds__(kWaves * 64)
void vocab_pass_kernel(VocabPassArgs a, int rpb)
{
    static_assert(kAhead >= 1 && kAhead <= kDepth && kDepth % kAhead == 0, "the register ring must close over a super-tile");
    static_assert(kWaves <= kMaxWaves, "one hint slot per wave");
    extern __shared__ __align__(16) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t V = a.V;
    const int nst = (int)((V + kSuperCols - 1) / kSuperCols);   // super-tiles in a row
    const int nfull = (int)(V / kSuperCols);                    // of which complete
    const int64_t row0 = (int64_t)blockIdx.x * rpb;             // first row of this workgroup
    const int nrows = (int)((a.rows - row0) < rpb ? (a.rows - row0) : rpb);
    // items: the rows' incomplete super-tiles first, then complete ones row by row
    const int n_ragged = nst > nfull ? nrows : 0;
    const int total = n_ragged + nrows * nfull;

    WaveHint* hints = reinterpret_cast<WaveHint*>(smem);
    uint32_t* done = reinterpret_cast<uint32_t*>(smem + sizeof(WaveHint) * kMaxWaves);
    RowPartial* parts = reinterpret_cast<RowPartial*>(smem + lds_done_bytes(rpb));
    float* inv_e_tab = reinterpret_cast<float*>(smem + lds_done_bytes(rpb)
                                                + sizeof(RowPartial) * (size_t)rpb * (kWaves + 1));

    const int64_t row_bytes = a.row_stride * (int64_t)Chunk::kElemBytes;
    const int64_t lane_col = (int64_t)lane * kChunk;            // own columns (incomplete sweeps)
    const int64_t sweep_lane_col = Chunk::sweep_col(lane);      // complete sweeps: see the loaders
    const int tlane = Chunk::tile_lane(lane);                   // tile lane held after unpack_sweep
    const char* base = static_cast<const char*>(a.logits) + row0 * row_bytes;

    // item -> (local row, super-tile)
    auto decode = [&](int item, int& r, int& st) {
        if (item < n_ragged) { r = item; st = nfull; }
        else { const int idx = item - n_ragged; r = idx / nfull; st = idx - r * nfull; }
    };

    // Wave w takes items w, w + kWaves, ...; if the first is a complete super-tile its
    // first sweeps are requested before anything else happens.
    int item = wave;
    bool have = item < total;
    Chunk buf[kAhead];
    int r_cur = 0, st_cur = 0;
    if (have && item >= n_ragged) {
        decode(item, r_cur, st_cur);
        const char* rp = base + r_cur * row_bytes;
        const int64_t b0 = (int64_t)st_cur * kSuperCols + sweep_lane_col;
#pragma unroll
        for (int i = 0; i < kAhead; ++i) buf[i].load_sweep(rp, b0 + i * kSweepCols);
    }

    // Workgroup prologue: empty hand-over slots, and (rollout side) the level-1 noise of all
    // tiles of the workgroup's rows, one Philox block per thread per four tiles.
    for (int i = threadIdx.x; i < rpb; i += kWaves * 64) done[i] = 0;
    for (int i = threadIdx.x; i < rpb * (kWaves + 1); i += kWaves * 64) {
        RowPartial e;
        e.S = 0.0; e.W = 0.0; e.rc = -INFINITY; e.top = -INFINITY; e.q = -1.0f; e.tile = 0;
        parts[i] = e;
    }
    if (kSample) {
        const uint32_t seed_lo = (uint32_t)a.seed, seed_hi = (uint32_t)(a.seed >> 32);
        const int calls = nrows * nst * (kLanes / 4);
        for (int cidx = threadIdx.x; cidx < calls; cidx += kWaves * 64) {
            const int r = cidx / (nst * 16), rem = cidx - r * (nst * 16);   // rem = tile / 4 in the row
            const uint64_t grow = a.row_base + (uint64_t)(row0 + r);
            uint32_t w[4];
            philox4x32_10((uint32_t)rem, (uint32_t)grow, (uint32_t)(grow >> 32), 1u, seed_lo, seed_hi, w);
            float4 v;
            v.x = inv_exp_variate(w[0]); v.y = inv_exp_variate(w[1]);
            v.z = inv_exp_variate(w[2]); v.w = inv_exp_variate(w[3]);
            reinterpret_cast<float4*>(inv_e_tab)[(size_t)r * nst * 16 + rem] = v;
        }
    }
    // Every wave whose first item is a complete super-tile tells the workgroup one logit value
    // that item's row holds: the largest among the sweeps it has requested (they have arrived
    // by now on the rollout side, behind the noise table).  The largest of these per row is
    // the floor the waves start that row with; it depends on the data and the launch shape only.
    {
        float mine = -INFINITY;
        int mine_row = -1;
        if (have && item >= n_ragged) {
#pragma unroll
            for (int i = 0; i < kAhead; ++i) mine = fmaxf(mine, buf[i].some_max());
            mine = wave_max(mine);
            mine_row = r_cur;
        }
        if (lane == 0) hints[wave] = WaveHint{mine_row, mine};
    }
    // Workgroup barrier that orders LDS only: __syncthreads() would also wait for the
    // global loads already in flight (its fence covers global memory) and drain the
    // pipeline for a full memory latency.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // floor of local row r: just below the largest hint given for it (-inf: none)
    auto row_floor = [&](int r) -> float {
        float v = -INFINITY;
        if (lane < kWaves) {
            const WaveHint h = hints[lane];
            if (h.row == r) v = h.value;
        }
        v = row16_max(v);
        return v > -INFINITY ? v - fmaxf(fabsf(v) * 0x1p-12f, 1.0e-30f) : -INFINITY;
    };

    // Training side, optional: rollout groups riding along.  The last wave has the fewest
    // items (or as many as the others), so it takes workgroup b's group b before it starts
    // on its own; the loads of its first item are already in flight.  The host asks for
    // this only when there are at most as many groups as workgroups.
    if (!kSample && a.adv_groups > 0 && wave == kWaves - 1 && (int)blockIdx.x < a.adv_groups)
        advantages_of_group(a.adv_rewards, a.adv_offsets, (int)blockIdx.x, a.adv_ddof, a.adv_eps,
                            a.adv_out, lane);

    // Hand over what this wave holds for local row r (n_items of its items); the wave
    // that brings the row's count to nst finishes the row.
    auto deliver = [&](LaneState& s, int r, int slot, int n_items) {
        const double Sw = wave_sum((double)s.S);
        const double Ww = wave_sum((double)s.W);
        const Cand wb = kSample ? wave_best(s.best) : Cand{-1.0f, 0};
        uint32_t before = 0;
        if (lane == 0) {
            RowPartial p;
            p.S = Sw; p.W = Ww; p.rc = s.rc; p.top = s.top; p.q = wb.q; p.tile = wb.idx;
            parts[r * (kWaves + 1) + slot] = p;
            // Release: the partial is visible to the workgroup before the counter moves.
            // The fence is restricted to the LDS address space, so it waits for this
            // wave's LDS operations only and leaves its global loads in flight.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            before = __hip_atomic_fetch_add(&done[r], (uint32_t)n_items, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        before = __builtin_amdgcn_readfirstlane(before);
        if ((int)before + n_items == nst) {
            // Acquire: the counter said every other wave's partial of this row is written;
            // order the reads of those partials behind it (LDS only, as above).
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            finish_row<Chunk, kSample, true>(a, row0 + r, parts + r * (kWaves + 1), kWaves + 1, lane);
        }
    };
    auto row_scale = [&](int r) -> float {
        const float tau = a.tau_rows ? a.tau_rows[row0 + r] : a.tau_scalar;
        return kLog2eF / tau;
    };

    // Incomplete super-tiles come first in the item order, so a wave meets them before it
    // enters the pipelined loop.
    while (have && item < n_ragged) {
        const int next = item + kWaves;
        const int r = item, st = nfull;
        const char* rowp = base + r * row_bytes;
        const float c = row_scale(r);
        const float inv_e = kSample ? inv_e_tab[((size_t)r * nst + st) * kLanes + lane] : 0.0f;
        LaneState s;
        start_row(s, row_floor(r), c);
        const bool any_valid = stream_ragged<Chunk>(s, rowp, (int64_t)st * kSuperCols + lane_col,
                                                    lane_col, V, c, lane);
        close_tile<kSample>(s, st * kLanes + lane, inv_e, any_valid, c, lane);
        deliver(s, r, kWaves, 1);
        item = next;
        have = item < total;
        if (have && item >= n_ragged) {
            decode(item, r_cur, st_cur);
            const char* rp = base + r_cur * row_bytes;
            const int64_t b0 = (int64_t)st_cur * kSuperCols + sweep_lane_col;
#pragma unroll
            for (int i = 0; i < kAhead; ++i) buf[i].load_sweep(rp, b0 + i * kSweepCols);
        }
    }

    if (have) {
        // Pipelined loop over complete super-tiles.  Invariant at the top: (r_cur, st_cur)
        // is a complete super-tile whose first kAhead sweeps are requested into buf.
        // Items come in increasing order, so the rows a wave sees never go back: it
        // accumulates one row in `s` and hands it over when the row changes.
        LaneState s;
        int held = 0;                                    // items of r_cur accumulated in s
        float c = row_scale(r_cur);
        start_row(s, row_floor(r_cur), c);
        const char* rowp = base + r_cur * row_bytes;
        while (true) {
            const int next = item + kWaves;
            const float inv_e = kSample ? inv_e_tab[((size_t)r_cur * nst + st_cur) * kLanes + tlane] : 0.0f;
            const int64_t this_base = (int64_t)st_cur * kSuperCols + sweep_lane_col;
#pragma unroll
            for (int i = 0; i < kDepth - kAhead; ++i) {
                float z[8];
                buf[i % kAhead].unpack_sweep(z, lane);
                buf[i % kAhead].load_sweep(rowp, this_base + (i + kAhead) * kSweepCols);
                accumulate_chunk(s, z, c, lane);
            }
            const bool more = next < total;
            int r_next = r_cur, st_next = 0;
            const char* nrowp = rowp;
            int64_t next_base = 0;
            if (more) {
                decode(next, r_next, st_next);
                nrowp = base + r_next * row_bytes;
                next_base = (int64_t)st_next * kSuperCols + sweep_lane_col;
            }
            // two copies of the last sweeps, with and without the requests for the next item:
            // a request under a condition inside one copy makes the compiler wait for more
            // of the loads in flight than the copy with requests needs to
            if (more) {
#pragma unroll
                for (int i = kDepth - kAhead; i < kDepth; ++i) {
                    float z[8];
                    buf[i % kAhead].unpack_sweep(z, lane);
                    buf[i % kAhead].load_sweep(nrowp, next_base + (i + kAhead - kDepth) * kSweepCols);
                    accumulate_chunk(s, z, c, lane);
                }
            } else {
#pragma unroll
                for (int i = kDepth - kAhead; i < kDepth; ++i) {
                    float z[8];
                    buf[i % kAhead].unpack_sweep(z, lane);
                    accumulate_chunk(s, z, c, lane);
                }
            }
            close_tile<kSample>(s, st_cur * kLanes + tlane, inv_e, true, c, lane);
            ++held;
            if (!more || r_next != r_cur) {
                deliver(s, r_cur, wave, held);
                held = 0;
            }
            if (!more) break;
            if (r_next != r_cur) {
                c = row_scale(r_next);
                rowp = base + r_next * row_bytes;
                start_row(s, row_floor(r_next), c);
            }
            r_cur = r_next;
            st_cur = st_next;
            item = next;
        }
    }
}

// ---------------------------------------------------------------------------
// Small batches.  When the rows are too few to give every compute unit a workgroup
// of whole rows, a row is cut into `nslots` runs of consecutive super-tiles and
// every run gets a one-wave workgroup of its own, so that all of the chip's memory
// channels are busy even for a single row.  A wave requests a whole super-tile (all
// kDepth sweeps) at once, refills each register with the same sweep of its next super-tile
// as soon as it has consumed it, draws the level-1 noise of its own tiles while the
// loads are in flight, and writes one RowPartial to the workspace.  A second launch
// of one wave per row merges a row's partials exactly as the row-block kernel's
// epilogue does.
// ---------------------------------------------------------------------------
template <typename Chunk, bool kSample>
__global__ __launch_bounds__(64)
void vocab_split_kernel(VocabPassArgs a, RowPartial* __restrict__ ws, int nslots)
{
    const int lane = threadIdx.x;
    const int64_t V = a.V;
    const int nst = (int)((V + kSuperCols - 1) / kSuperCols);
    const int nfull = (int)(V / kSuperCols);
    const int64_t row = (int64_t)blockIdx.x / nslots;
    const int slot = (int)((int64_t)blockIdx.x - row * nslots);
    const int st_begin = slot * nst / nslots;        // runs differ by at most one super-tile
    const int st_end = (slot + 1) * nst / nslots;

    const char* rowp = static_cast<const char*>(a.logits) + row * a.row_stride * (int64_t)Chunk::kElemBytes;
    const int64_t lane_col = (int64_t)lane * kChunk;            // own columns (incomplete sweeps)
    const int64_t sweep_lane_col = Chunk::sweep_col(lane);      // complete sweeps: see the loaders
    const int tlane = Chunk::tile_lane(lane);

    Chunk buf[kDepth];
    if (st_begin < nfull) {
        const int64_t b0 = (int64_t)st_begin * kSuperCols + sweep_lane_col;
#pragma unroll
        for (int i = 0; i < kDepth; ++i) buf[i].load_sweep(rowp, b0 + i * kSweepCols);
    }
    const float tau = a.tau_rows ? a.tau_rows[row] : a.tau_scalar;
    const float c = kLog2eF / tau;
    const uint64_t grow = a.row_base + (uint64_t)row;

    LaneState s;
    start_row(s, -INFINITY, c);
    for (int st = st_begin; st < st_end; ++st) {
        const int tile = st * kLanes + (st < nfull ? tlane : lane);
        float inv_e = 0.0f;
        if (kSample) {
            uint32_t w[4];
            philox4x32_10((uint32_t)(tile >> 2), (uint32_t)grow, (uint32_t)(grow >> 32), 1u,
                          (uint32_t)a.seed, (uint32_t)(a.seed >> 32), w);
            const int k = tile & 3;
            inv_e = inv_exp_variate(k == 0 ? w[0] : k == 1 ? w[1] : k == 2 ? w[2] : w[3]);
        }
        if (st < nfull) {
            const bool refill = st + 1 < st_end && st + 1 < nfull;     // uniform
            const int64_t nb = (int64_t)(st + 1) * kSuperCols + sweep_lane_col;
#pragma unroll
            for (int i = 0; i < kDepth; ++i) {
                float z[8];
                buf[i].unpack_sweep(z, lane);
                if (refill) buf[i].load_sweep(rowp, nb + i * kSweepCols);
                accumulate_chunk(s, z, c, lane);
            }
            close_tile<kSample>(s, tile, inv_e, true, c, lane);
        } else {
            const bool any_valid = stream_ragged<Chunk>(s, rowp, (int64_t)st * kSuperCols + lane_col,
                                                        lane_col, V, c, lane);
            close_tile<kSample>(s, tile, inv_e, any_valid, c, lane);
        }
    }
    const double Sw = wave_sum((double)s.S);
    const double Ww = wave_sum((double)s.W);
    const Cand wb = kSample ? wave_best(s.best) : Cand{-1.0f, 0};
    if (lane == 0) {
        RowPartial p;
        p.S = Sw; p.W = Ww; p.rc = s.rc; p.top = s.top; p.q = wb.q; p.tile = wb.idx;
        ws[(size_t)blockIdx.x] = p;
    }
}

template <typename Chunk, bool kSample>
__global__ __launch_bounds__(64)
void row_finish_kernel(VocabPassArgs a, const RowPartial* __restrict__ ws, int nslots)
{
    finish_row<Chunk, kSample, false>(a, (int64_t)blockIdx.x, ws + (size_t)blockIdx.x * nslots, nslots,
                                      (int)threadIdx.x);
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
constexpr size_t kLdsBudget = 64 * 1024;

// Optional events for the next vocabulary-pass launch of this host thread: `start` gets
// the time the (first) kernel begins to execute, `stop` the time the (last) kernel ends,
// taken from the dispatch itself rather than from marker packets around it.
static thread_local hipEvent_t g_start_event = nullptr;
static thread_local hipEvent_t g_stop_event = nullptr;

void set_launch_events(hipEvent_t start, hipEvent_t stop)
{
    g_start_event = start;
    g_stop_event = stop;
}

LaunchEvents take_launch_events()
{
    LaunchEvents e{g_start_event, g_stop_event};
    g_start_event = nullptr;
    g_stop_event = nullptr;
    return e;
}

// Rows per workgroup: at least two items per wave (one row of 38 super-tiles at
// V = 151,936 gives a wave 4 or 5), and the noise table must fit LDS
// (0 = does not fit).  Two 8-wave workgroups are resident per compute unit; what exceeds
// that is handed out by the hardware dispatcher as workgroups finish.
template <int kWaves>
static int rows_per_group(int64_t V, bool sample)
{
    const int nst = (int)((V + kSuperCols - 1) / kSuperCols);
    int rpb = (2 * kWaves + nst - 1) / nst;
    if (rpb < 1) rpb = 1;
    while (rpb > 1 && lds_bytes<kWaves>(rpb, nst, sample) > kLdsBudget) --rpb;
    if (lds_bytes<kWaves>(rpb, nst, sample) > kLdsBudget) return 0;
    return rpb;
}

bool vocab_pass_fits(int64_t V) { return rows_per_group<8>(V, true) > 0 && rows_per_group<4>(V, true) > 0; }

static int compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

template <typename Chunk, bool kSample, int kWaves>
static hipError_t launch_groups(const VocabPassArgs& a, hipStream_t stream)
{
    const int rpb = rows_per_group<kWaves>(a.V, kSample);
    if (rpb == 0) return hipErrorInvalidValue;
    const int nst = (int)((a.V + kSuperCols - 1) / kSuperCols);
    const size_t lds = lds_bytes<kWaves>(rpb, nst, kSample);
    const unsigned blocks = (unsigned)((a.rows + rpb - 1) / rpb);
    const LaunchEvents ev = take_launch_events();
    if (ev.start != nullptr || ev.stop != nullptr)
        hipExtLaunchKernelGGL((vocab_pass_kernel<Chunk, kSample, kWaves, Chunk::kAhead>),
                              dim3(blocks), dim3(kWaves * 64), (uint32_t)lds, stream, ev.start, ev.stop, 0u,
                              a, rpb);
    else
        hipLaunchKernelGGL((vocab_pass_kernel<Chunk, kSample, kWaves, Chunk::kAhead>),
                           dim3(blocks), dim3(kWaves * 64), lds, stream, a, rpb);
    return hipGetLastError();
}

// Eight waves per workgroup while the whole batch is at most eight workgroups per
// compute unit; four waves per workgroup beyond that, where the hardware dispatcher
// balances across many small groups (measured crossover on MI355X: between 2048 and
// 4096 rows of 151,936 bf16 columns).  Two 8-wave workgroups are resident per compute
// unit: a batch that fills its last round of 2 * CUs workgroups to less than 80 %
// (768 rows on 256 CUs: 512 + 256) runs as 4-wave workgroups if those are all resident
// at once (measured at 768 rows: 45.0 us instead of 49.3 us).
template <typename Chunk, bool kSample>
static hipError_t launch_for(const VocabPassArgs& a, hipStream_t stream)
{
#ifdef E3_FORCE_WAVES
    return launch_groups<Chunk, kSample, E3_FORCE_WAVES>(a, stream);
#else
    const int64_t cus = compute_units();
    const int rpb8 = rows_per_group<8>(a.V, kSample);
    const int rpb4 = rows_per_group<4>(a.V, kSample);
    if (rpb8 == 0) return launch_groups<Chunk, kSample, 4>(a, stream);
    const int64_t groups8 = (a.rows + rpb8 - 1) / rpb8;
    if (groups8 > 8 * cus) return launch_groups<Chunk, kSample, 4>(a, stream);
    const int64_t round8 = 2 * cus;
    const int64_t rounds = (groups8 + round8 - 1) / round8;
    if (groups8 > round8 && groups8 * 5 < rounds * round8 * 4 && rpb4 > 0
        && (a.rows + rpb4 - 1) / rpb4 <= 4 * cus)
        return launch_groups<Chunk, kSample, 4>(a, stream);
    return launch_groups<Chunk, kSample, 8>(a, stream);
#endif
}

// Split path: used when the row-block path would leave compute units without a
// workgroup and the caller brought enough workspace.  Every super-tile gets a wave of
// its own (measured on MI355X: one-wave workgroups beyond what is resident are handed
// out by the hardware dispatcher as earlier ones finish, which balances better than
// longer static runs), except that a row has at most 64 runs: one partial per lane
// of the merging wave.
constexpr int64_t kSplitMaxRows = 1024;          // bound used by the workspace size

struct SplitPlan {
    int nslots;      // runs per row, 1 <= nslots <= min(64, super-tiles per row)
};

static SplitPlan split_plan(int64_t V)
{
    const int nst = (int)((V + kSuperCols - 1) / kSuperCols);
    SplitPlan p;
    p.nslots = nst < 64 ? nst : 64;
    return p;
}

size_t vocab_pass_workspace_bytes(int64_t rows, int64_t V)
{
    if (rows <= 0 || rows > kSplitMaxRows || V <= 0) return 0;
    const int64_t nst = (V + kSuperCols - 1) / kSuperCols;
    return (size_t)rows * (size_t)(nst < 64 ? nst : 64) * sizeof(RowPartial);
}

template <typename Chunk, bool kSample>
static hipError_t launch_split(const VocabPassArgs& a, RowPartial* ws, SplitPlan plan, hipStream_t stream)
{
    const unsigned blocks = (unsigned)(a.rows * plan.nslots);
    const LaunchEvents ev = take_launch_events();
    const RowPartial* parts = ws;
    if (ev.start != nullptr)
        hipExtLaunchKernelGGL((vocab_split_kernel<Chunk, kSample>), dim3(blocks), dim3(64), 0u, stream,
                              ev.start, (hipEvent_t) nullptr, 0u, a, ws, plan.nslots);
    else
        hipLaunchKernelGGL((vocab_split_kernel<Chunk, kSample>), dim3(blocks), dim3(64), 0, stream,
                           a, ws, plan.nslots);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (ev.stop != nullptr)
        hipExtLaunchKernelGGL((row_finish_kernel<Chunk, kSample>), dim3((unsigned)a.rows), dim3(64), 0u,
                              stream, (hipEvent_t) nullptr, ev.stop, 0u, a, parts, plan.nslots);
    else
        hipLaunchKernelGGL((row_finish_kernel<Chunk, kSample>), dim3((unsigned)a.rows), dim3(64), 0, stream,
                           a, parts, plan.nslots);
    return hipGetLastError();
}

// Number of workgroups the row-block launch of this shape will have (both wave counts
// give the same number when a workgroup holds one row).
template <int kWaves>
static int64_t row_block_groups(int64_t rows, int64_t V, bool sample)
{
    const int rpb = rows_per_group<kWaves>(V, sample);
    return rpb > 0 ? (rows + rpb - 1) / rpb : 0;
}

hipError_t launch_vocab_pass(const VocabPassArgs& args, bool is_bf16, bool sample,
                             void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    VocabPassArgs a = args;
    // Groups ride along only in a row-block launch that has a workgroup for each of them
    // with either wave count; otherwise they get their own launch first.
    auto separate_advantages = [&]() -> hipError_t {
        const hipError_t err = launch_grpo_advantages(a.adv_rewards, a.adv_offsets, a.adv_groups,
                                                      a.adv_ddof, a.adv_eps, a.adv_out, stream);
        a.adv_groups = 0;
        return err;
    };
    if (a.adv_groups > 0 && a.rows == 0) return separate_advantages();
    if (a.rows == 0) return hipSuccess;
    const int cus = compute_units();
    const int rpb8 = rows_per_group<8>(a.V, sample);
#ifdef E3_SPLIT_ALWAYS
    const bool few = a.rows <= kSplitMaxRows;
#else
    const bool few = a.rows <= kSplitMaxRows && rpb8 > 0
                  && (a.rows + rpb8 - 1) / rpb8 * E3_SPLIT_BELOW_DEN <= (int64_t)cus * E3_SPLIT_BELOW_NUM;
#endif
    if (few && workspace != nullptr && (reinterpret_cast<uintptr_t>(workspace) & 15u) == 0) {
        const SplitPlan plan = split_plan(a.V);
        if ((size_t)a.rows * plan.nslots * sizeof(RowPartial) <= workspace_bytes) {
            RowPartial* ws = static_cast<RowPartial*>(workspace);
            if (a.adv_groups > 0) {
                const hipError_t err = separate_advantages();
                if (err != hipSuccess) return err;
            }
            if (is_bf16)
                return sample ? launch_split<ChunkBf16, true>(a, ws, plan, stream)
                              : launch_split<ChunkBf16, false>(a, ws, plan, stream);
            return sample ? launch_split<ChunkF32, true>(a, ws, plan, stream)
                          : launch_split<ChunkF32, false>(a, ws, plan, stream);
        }
    }
    if (a.adv_groups > 0) {
        const int64_t g8 = row_block_groups<8>(a.rows, a.V, sample), g4 = row_block_groups<4>(a.rows, a.V, sample);
        if (sample || a.adv_groups > g8 || a.adv_groups > g4) {
            const hipError_t err = separate_advantages();
            if (err != hipSuccess) return err;
        }
    }
    if (is_bf16)
        return sample ? launch_for<ChunkBf16, true>(a, stream)
                      : launch_for<ChunkBf16, false>(a, stream);
    return sample ? launch_for<ChunkF32, true>(a, stream)
                  : launch_for<ChunkF32, false>(a, stream);
}

// ---------------------------------------------------------------------------
// Library-owned scratch for callers that cannot allocate: the small-batch path's row
// partials in a file-scope device array instead of a caller workspace.  Every GPU the
// library runs on holds its own copy of the array at its own address, looked up once
// per device; host code uses that address, never the array's name.
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)kSplitMaxRows * 64 * sizeof(RowPartial);   // 2 MiB
static_assert(kStaticScratchBytes == 2u * 1024 * 1024, "documented size");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

int64_t static_scratch_max_rows() { return kSplitMaxRows; }

hipError_t static_scratch(void** ptr_out, size_t* bytes_out)
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));     // this device's copy
        if (err != hipSuccess) return err;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr_out = g_scratch_ptr[dev];
    *bytes_out = kStaticScratchBytes;
    return hipSuccess;
}

hipError_t launch_entropy_reduce(const float* entropy, const uint8_t* mask, int64_t rows,
                                 double* sum_out, int64_t* count_out, hipStream_t stream,
                                 hipEvent_t stop_event)
{
    if (stop_event != nullptr)
        hipExtLaunchKernelGGL(entropy_reduce_kernel, dim3(1), dim3(1024), 0u, stream,
                              (hipEvent_t) nullptr, stop_event, 0u, entropy, mask, rows, sum_out, count_out);
    else
        hipLaunchKernelGGL(entropy_reduce_kernel, dim3(1), dim3(1024), 0, stream,
                           entropy, mask, rows, sum_out, count_out);
    return hipGetLastError();
}

}  // namespace e3
