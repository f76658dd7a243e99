// Persistent streaming form of the vocabulary pass (gfx950).
//
// The [rows, V] logit matrix is cut into work items of one super-tile (8192 columns
// of one row = 16 KiB of bf16).  A fixed set of single-wave workgroups, a few per
// SIMD, pulls items from a device-side counter, so that every wave keeps streaming
// until the whole matrix is consumed no matter how unevenly the memory system serves
// them; a wave keeps the first sweeps of its next item in flight while it finishes
// the current one.  Each item leaves a 32-byte partial (reference, excluded maximum,
// sums, best sampler tile); the wave that delivers the last partial of a row merges
// them, runs level 2 of the sampler and writes the row's outputs.
//
// What is computed is the same as in vocab_pass.hip (Appendix A of arXiv 2505.18573:
// temperature softmax, entropy through H = ln S - W/S; two-level Gumbel-max as
// specified in include/e3.h); only the decomposition of the work differs.
//
// Workspace (zero-filled before first use; every launch leaves it zero-filled):
//   [0, 64)                    StreamHeader: item counter, exit counter
//   [64, 64 + 4*rows_pad)      per-row count of delivered partials
//   then                       TilePartial[rows * nst]
#include "vocab_common.h"
#include "vocab_pass.h"

namespace e3 {

struct alignas(16) TilePartial {
    double S, W;       // sums over the item's columns except `top`, relative to rc
    float rc, top;     // reference and excluded maximum
    float q;           // mass / E of the item's best sampler tile, relative to rc
    int tile;          // its tile id
};
static_assert(sizeof(TilePartial) == 32, "layout");

struct StreamHeader {
    uint32_t next_ticket;   // dynamic items handed out so far
    uint32_t exited;        // waves that have left the item loop
    uint32_t pad[14];
};
static_assert(sizeof(StreamHeader) == 64, "layout");

__host__ __device__ inline size_t stream_rows_pad(int64_t rows) { return (size_t)((rows + 15) / 16 * 16); }

size_t stream_workspace_bytes(int64_t rows, int64_t V)
{
    const int64_t nst = (V + kSuperCols - 1) / kSuperCols;
    return sizeof(StreamHeader) + 4 * stream_rows_pad(rows) + sizeof(TilePartial) * (size_t)(rows * nst);
}

__device__ __forceinline__ uint32_t agent_fetch_add(uint32_t* p, uint32_t v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Row epilogue, run by the wave that delivered the row's last partial: merge the
// partials (one per lane), level 2 of the sampler or the target gather, outputs.
template <typename Chunk, bool kSample>
__device__ __forceinline__ void finish_row(const VocabPassArgs& a, int64_t row, int nst,
                                           TilePartial* parts, uint32_t* row_count, int lane)
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

    TilePartial p;
    p.S = 0.0; p.W = 0.0; p.rc = -INFINITY; p.top = -INFINITY; p.q = -1.0f; p.tile = 0;
    TilePartial* mine = parts + row * nst + lane;
    if (lane < nst) {
        p = *mine;
        TilePartial zero;
        zero.S = 0.0; zero.W = 0.0; zero.rc = 0.0f; zero.top = 0.0f; zero.q = 0.0f; zero.tile = 0;
        *mine = zero;                                   // leave the workspace clean
    }
    if (lane == 0) row_count[row] = 0;

    // R is the common reference, `peak` the largest logit of the row; the partial
    // that holds it is the lowest lane with that top, every other excluded maximum
    // joins the rest as an ordinary term.  All in fp64 from here.
    const float R = wave_max(p.rc);
    const float peak = wave_max(p.top);
    const unsigned long long holders = __ballot(p.top == peak);
    const int peak_lane = (int)__builtin_ctzll(holders | (1ull << 63));
    const bool live = p.rc > -INFINITY;
    const double cd = (double)c;
    const double d = live ? (double)R - (double)p.rc : 0.0;       // integer >= 0
    const int sh = d > 4000.0 ? -4000 : -(int)d;
    double S_l = 0.0, W_l = 0.0;
    if (live) {
        S_l = ldexp(p.S, sh);
        W_l = ldexp(p.W - d * p.S, sh);
        if (lane != peak_lane) {
            const double tw = (double)p.top * cd - (double)R;
            const double ew = (double)exp2f((float)tw);
            S_l += ew;
            W_l += tw * ew;
        }
    }
    const double S_rest = wave_sum(S_l);
    const double W_rest = wave_sum(W_l);
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
        // level 1 across items: weights brought to the common reference (exact scaling)
        Cand cand{live ? ldexpf(p.q, sh) : -1.0f, p.tile};
        const Cand win = wave_best(cand);
        // Level 2: Gumbel-max inside the winning tile, in race form: maximise
        // 2^{(z - zmax) c} / E_col.  32 lanes x 4 consecutive columns cover the tile.
        const int wst = win.idx / kLanes, wslot = win.idx % kLanes;
        const int64_t col0 = (int64_t)wst * kSuperCols + (int64_t)(lane >> 1) * kSweepCols
                           + (int64_t)wslot * kChunk + (lane & 1) * 4;
        float cz[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            cz[j] = (lane < 32 && col0 + j < V) ? Chunk::load_one(rowp, col0 + j) : kAbsent;
        const uint64_t grow = a.row_base + (uint64_t)row;
        uint32_t w[4];
        philox4x32_10((uint32_t)(col0 >> 2), (uint32_t)grow, (uint32_t)(grow >> 32), 2u,
                      (uint32_t)a.seed, (uint32_t)(a.seed >> 32), w);
        const float zmax = wave_max(fmaxf(fmaxf(cz[0], cz[1]), fmaxf(cz[2], cz[3])));
        Cand cb{-1.0f, 0x7FFFFFFF};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool ok = lane < 32 && col0 + j < V;
            const float q = __builtin_amdgcn_exp2f((cz[j] - zmax) * c) / exp_variate(w[j]);
            cb = better(cb, Cand{ok ? q : -1.0f, ok ? (int)(col0 + j) : 0x7FFFFFFF});
        }
        cb = wave_best(cb);
        tok = cb.idx;
        if (tok < 0 || tok >= V) tok = 0;                 // only reachable with non-finite input
        float own = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (col0 + j == tok) own = cz[j];
        z_tok = wave_max(own);
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

template <typename Chunk, bool kSample, int kAhead>
__global__ __launch_bounds__(64)
void vocab_stream_kernel(VocabPassArgs a, char* ws)
{
    static_assert(kAhead >= 1 && kAhead < kDepth, "the follow-up item must be known mid-item");
    const int lane = threadIdx.x;
    const int64_t V = a.V;
    const int nst = (int)((V + kSuperCols - 1) / kSuperCols);
    const int nfull = (int)(V / kSuperCols);
    const uint32_t n_ragged = nst > nfull ? (uint32_t)a.rows : 0u;   // ragged items come first
    const uint32_t total = n_ragged + (uint32_t)a.rows * (uint32_t)nfull;
    const uint32_t G = gridDim.x;

    StreamHeader* hdr = reinterpret_cast<StreamHeader*>(ws);
    uint32_t* row_count = reinterpret_cast<uint32_t*>(ws + sizeof(StreamHeader));
    TilePartial* parts = reinterpret_cast<TilePartial*>(ws + sizeof(StreamHeader)
                                                        + 4 * stream_rows_pad(a.rows));
    const uint32_t seed_lo = (uint32_t)a.seed, seed_hi = (uint32_t)(a.seed >> 32);
    const int64_t row_bytes = a.row_stride * (int64_t)Chunk::kElemBytes;
    const int64_t lane_col = (int64_t)lane * kChunk;

    // item -> (row, super-tile)
    auto decode = [&](uint32_t item, int64_t& row, int& st) {
        if (item < n_ragged) { row = item; st = nfull; }
        else { const uint32_t idx = item - n_ragged; row = idx / (uint32_t)nfull; st = (int)(idx % (uint32_t)nfull); }
    };
    auto take_ticket = [&]() -> uint32_t {
        uint32_t t = 0;
        if (lane == 0) t = agent_fetch_add(&hdr->next_ticket, 1u);
        return t;                                        // valid in lane 0
    };

    // Deliver one item's result; the wave that completes a row finishes it.
    auto deliver = [&](LaneState& s, int64_t row, int st) {
        const double Sw = wave_sum((double)s.S);
        const double Ww = wave_sum((double)s.W);
        const Cand wb = kSample ? wave_best(s.best) : Cand{-1.0f, 0};
        uint32_t before = 0;
        if (lane == 0) {
            TilePartial p;
            p.S = Sw; p.W = Ww; p.rc = s.rc; p.top = s.top; p.q = wb.q; p.tile = wb.idx;
            parts[row * nst + st] = p;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        if (lane == 0) before = agent_fetch_add(&row_count[row], 1u);
        before = __builtin_amdgcn_readfirstlane(before);
        if (before == (uint32_t)(nst - 1)) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            finish_row<Chunk, kSample>(a, row, nst, parts, row_count, lane);
        }
    };

    auto tile_noise = [&](int64_t row, int st) -> float {
        if (!kSample) return 0.0f;
        const uint64_t grow = a.row_base + (uint64_t)row;
        uint32_t w[4];
        philox4x32_10((uint32_t)(st * 16 + (lane >> 2)), (uint32_t)grow, (uint32_t)(grow >> 32), 1u,
                      seed_lo, seed_hi, w);
        const uint32_t pick = (lane & 2) ? ((lane & 1) ? w[3] : w[2]) : ((lane & 1) ? w[1] : w[0]);
        return 1.0f / exp_variate(pick);
    };

    auto fresh = [&](LaneState& s) {
        s.rc = -INFINITY; s.top = -INFINITY; s.dom_lane = 0; s.dom_open = false;
        s.S = s.W = s.sT0 = s.sT1 = s.wT0 = s.wT1 = 0.0f;
        s.best = Cand{-1.0f, 0};
    };

    uint32_t item = blockIdx.x;                          // the first item is static
    bool have = item < total;

    // A wave whose first item is an incomplete super-tile does it before joining the
    // pipelined loop: sweeps in two halves of 8, guarded loads of a half all issued
    // before the first is used.
    while (have && item < n_ragged) {
        const uint32_t ticket = take_ticket();
        const int64_t row = item;
        const int st = nfull;
        const char* rowp = static_cast<const char*>(a.logits) + row * row_bytes;
        const float tau = a.tau_rows ? a.tau_rows[row] : a.tau_scalar;
        const float c = kLog2eF / tau;
        const float inv_e = tile_noise(row, st);
        LaneState s;
        fresh(s);
        const int64_t base = (int64_t)st * kSuperCols + lane_col;
        bool any_valid = false;
#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            const int64_t hbase = base + (int64_t)half * (kDepth / 2) * kSweepCols;
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
        close_tile<kSample>(s, st * kLanes + lane, inv_e, any_valid, c, lane);
        deliver(s, row, st);
        item = G + __builtin_amdgcn_readfirstlane(ticket);
        have = item < total;
    }

    if (have) {
        // Pipelined loop over complete super-tiles.  Invariant at the top: `item` is a
        // complete super-tile and its first kAhead sweeps are requested into buf.
        Chunk buf[kAhead];
        int64_t row;
        int st;
        decode(item, row, st);
        const char* rowp = static_cast<const char*>(a.logits) + row * row_bytes;
        {
            const int64_t b0 = (int64_t)st * kSuperCols + lane_col;
#pragma unroll
            for (int i = 0; i < kAhead; ++i) buf[i].load(rowp, b0 + i * kSweepCols);
        }
        float tau = a.tau_rows ? a.tau_rows[row] : a.tau_scalar;
        while (true) {
            const uint32_t ticket = take_ticket();       // answer needed kDepth - kAhead sweeps on
            const float c = kLog2eF / tau;
            const float inv_e = tile_noise(row, st);
            LaneState s;
            fresh(s);
            const int64_t this_base = (int64_t)st * kSuperCols + lane_col;
#pragma unroll
            for (int i = 0; i < kDepth - kAhead; ++i) {
                float z[8];
                buf[i % kAhead].unpack(z);
                buf[i % kAhead].load(rowp, this_base + (i + kAhead) * kSweepCols);
                accumulate_chunk(s, z, c, lane);
            }
            // the follow-up item; only a complete super-tile can be requested ahead
            const uint32_t next = G + __builtin_amdgcn_readfirstlane(ticket);
            const bool more = next < total;
            const bool ahead = more && next >= n_ragged;
            int64_t nrow = 0;
            int nst_ = 0;
            const char* nrowp = rowp;
            float ntau = tau;
            if (ahead) {
                decode(next, nrow, nst_);
                nrowp = static_cast<const char*>(a.logits) + nrow * row_bytes;
                ntau = a.tau_rows ? a.tau_rows[nrow] : a.tau_scalar;
            }
            if (ahead) {
                const int64_t next_base = (int64_t)nst_ * kSuperCols + lane_col;
#pragma unroll
                for (int i = kDepth - kAhead; i < kDepth; ++i) {
                    float z[8];
                    buf[i % kAhead].unpack(z);
                    buf[i % kAhead].load(nrowp, next_base + (i + kAhead - kDepth) * kSweepCols);
                    accumulate_chunk(s, z, c, lane);
                }
            } else {
#pragma unroll
                for (int i = kDepth - kAhead; i < kDepth; ++i) {
                    float z[8];
                    buf[i % kAhead].unpack(z);
                    accumulate_chunk(s, z, c, lane);
                }
            }
            close_tile<kSample>(s, st * kLanes + lane, inv_e, true, c, lane);
            deliver(s, row, st);
            if (!ahead) { item = next; have = more; break; }
            item = next; row = nrow; st = nst_; rowp = nrowp; tau = ntau;
        }
    }
    // `have` can only still be set here if a ragged item was handed out after the first
    // round (more rows than waves): take those one by one, unpipelined.
    while (have) {
        const uint32_t ticket = take_ticket();
        int64_t row;
        int st;
        decode(item, row, st);
        const char* rowp = static_cast<const char*>(a.logits) + row * row_bytes;
        const float tau = a.tau_rows ? a.tau_rows[row] : a.tau_scalar;
        const float c = kLog2eF / tau;
        const float inv_e = tile_noise(row, st);
        LaneState s;
        fresh(s);
        const int64_t base = (int64_t)st * kSuperCols + lane_col;
        bool any_valid = false;
#pragma unroll 1
        for (int i = 0; i < kDepth; ++i) {
            const int64_t col = base + i * kSweepCols;
            if (col - lane_col >= V) break;              // uniform
            float z[8];
            bool valid = false;
            if (col + kChunk <= V) {
                Chunk one;
                one.load(rowp, col);
                one.unpack(z);
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
        close_tile<kSample>(s, st * kLanes + lane, inv_e, any_valid, c, lane);
        deliver(s, row, st);
        item = G + __builtin_amdgcn_readfirstlane(ticket);
        have = item < total;
    }

    // The last wave out rewinds the counters for the next launch.
    if (lane == 0) {
        const uint32_t gone = agent_fetch_add(&hdr->exited, 1u);
        if (gone == G - 1) { hdr->next_ticket = 0; hdr->exited = 0; }
    }
}

__global__ void zero_words_kernel(uint32_t* p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

hipError_t launch_workspace_zero(void* ws, size_t bytes, hipStream_t stream)
{
    const size_t words = bytes / 4;
    if (words == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((words + 255) / 256 > 2048 ? 2048 : (words + 255) / 256);
    hipLaunchKernelGGL(zero_words_kernel, dim3(blocks), dim3(256), 0, stream,
                       static_cast<uint32_t*>(ws), words);
    return hipGetLastError();
}

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

#ifndef E3_STREAM_WAVES_PER_CU
#define E3_STREAM_WAVES_PER_CU 16
#endif
#ifndef E3_STREAM_AHEAD
#define E3_STREAM_AHEAD 8
#endif

bool stream_form_applies(const VocabPassArgs& a)
{
#ifndef E3_USE_STREAM
    (void)a;
    return false;
#else
    const int64_t nst = (a.V + kSuperCols - 1) / kSuperCols;
    const int64_t nfull = a.V / kSuperCols;
    // needs at least one complete super-tile per row, one lane per partial in the row
    // merge, and item ids that fit the 32-bit counter
    return nfull >= 1 && nst <= kLanes && a.rows * nst < (int64_t)0x7FFF0000;
#endif
}

template <typename Chunk, bool kSample>
static hipError_t launch_stream_for(const VocabPassArgs& a, void* ws, hipStream_t stream)
{
    const int64_t nst = (a.V + kSuperCols - 1) / kSuperCols;
    const int64_t total = a.rows * nst;
    int64_t waves = (int64_t)compute_units() * E3_STREAM_WAVES_PER_CU;
    if (waves > total) waves = total;
    hipLaunchKernelGGL((vocab_stream_kernel<Chunk, kSample, E3_STREAM_AHEAD>), dim3((unsigned)waves),
                       dim3(64), 0, stream, a, static_cast<char*>(ws));
    return hipGetLastError();
}

hipError_t launch_vocab_stream(const VocabPassArgs& a, bool is_bf16, bool sample, void* ws,
                               hipStream_t stream)
{
    if (a.rows == 0) return hipSuccess;
    if (is_bf16)
        return sample ? launch_stream_for<ChunkBf16, true>(a, ws, stream)
                      : launch_stream_for<ChunkBf16, false>(a, ws, stream);
    return sample ? launch_stream_for<ChunkF32, true>(a, ws, stream)
                  : launch_stream_for<ChunkF32, false>(a, ws, stream);
}

}  // namespace e3
