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
#include "vocab_common.h"
#include "vocab_pass.h"

namespace e3 {

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
