// Alloc-T selection and expert-sorted dispatch, as one single-workgroup "plan"
// kernel (the data is a few hundred KB at most and lives in L2).
//
// Selection (Section 3.3, Eqs. (7)-(9) and the procedure after them): every
// token keeps ranks j < K_base of its sorted candidate row; of the pool of the
// remaining T*(K-K_base) candidates the B' = B - T*K_base largest are kept,
// ties to the lower (token, rank).  Because rows are sorted, the kept ranks of
// a token form a prefix, so the result is keep_count[t].
//
// The B'-th largest pool value is found exactly by narrowing a range [lo, hi]
// of order-preserving u32 keys: each pass histograms the keys inside the range
// into <= 2048 equal-width bins in LDS (integer counts: order of the atomic
// increments cannot change the result), a block-wide suffix scan picks the bin
// that holds the wanted rank, and the range shrinks to that bin until it holds
// one key value v*.  Then a candidate is kept iff key > v*, or key == v* and
// fewer than R equal keys precede it in (token, rank) order.
//
// Dispatch: rows of the kept pairs ordered by (expert, token), with no atomics:
// for each batch of 64 tokens (lane = token) and each expert e the wave ballot
// "token keeps e" is a 64-bit word M[e][batch]; the row of pair (t, e) is
//   offset[e] + (kept pairs of e in earlier batches) + popcount(M[e][batch] below lane t).
#include <algorithm>

#include "common.hpp"
#include "kernels.hpp"

namespace allocmoe {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / kWave;
constexpr int kBinsLog2 = 11;
constexpr int kBins = 1 << kBinsLog2;

struct PlanShared {
    uint32_t hist[kBins];
    uint32_t wave_tot[kPlanWaves];
    uint32_t red_lo[kPlanWaves];
    uint32_t red_hi[kPlanWaves];
    uint32_t pick_bin;     // chosen bin of a pass
    uint32_t pick_rank;    // wanted rank inside the chosen bin
    uint32_t pick_count;   // number of keys inside the chosen bin
    int32_t expert_total[kWave];
    int32_t expert_off[kWave + 1];
};

// Exclusive block-wide prefix sum of one value per thread, in thread order.
// Returns the exclusive prefix; *total (optional) receives the block sum.
template <int NW = kPlanWaves>
__device__ __forceinline__ uint32_t block_scan_excl(uint32_t v, uint32_t* wave_tot,
                                                    uint32_t* total) {
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const uint32_t incl = static_cast<uint32_t>(wave_scan_incl(static_cast<int>(v)));
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t base = 0, sum = 0;
    for (int w = 0; w < NW; ++w) {
        const uint32_t x = wave_tot[w];
        if (w < wave) base += x;
        sum += x;
    }
    if (total) *total = sum;
    __syncthreads();
    return base + incl - v;
}

// keep_count[t] for all t.  topk_s: [T,K] rows sorted descending.
__device__ void select_phase(PlanShared& sh, const float* topk_s, int T, int K, int Kb,
                             int64_t B, int32_t* keep_count) {
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
    const int P = K - Kb;                       // pool entries per token
    const int64_t n_pool = static_cast<int64_t>(T) * P;
    const int64_t want = B - static_cast<int64_t>(T) * Kb;   // B'
    if (want <= 0 || want >= n_pool) {          // nothing or everything from the pool
        const int c = want <= 0 ? Kb : K;
        for (int t = tid; t < T; t += kPlanThreads) keep_count[t] = c;
        return;
    }

    if (tid == 0) {
        sh.pick_bin = 0;
        sh.pick_rank = 1;
        sh.pick_count = 1;
    }
    // ---- pass 0: range of the pool keys
    uint32_t lo = 0xFFFFFFFFu, hi = 0u;
    for (int t = tid; t < T; t += kPlanThreads)
        for (int j = Kb; j < K; ++j) {
            const uint32_t k = ordered_key(topk_s[static_cast<size_t>(t) * K + j]);
            lo = min(lo, k);
            hi = max(hi, k);
        }
    lo = wave_min_u32(lo);
    hi = wave_max_u32(hi);
    if (lane == 0) {
        sh.red_lo[wave] = lo;
        sh.red_hi[wave] = hi;
    }
    __syncthreads();
    lo = 0xFFFFFFFFu;
    hi = 0u;
    for (int w = 0; w < kPlanWaves; ++w) {
        lo = min(lo, sh.red_lo[w]);
        hi = max(hi, sh.red_hi[w]);
    }
    __syncthreads();

    // ---- narrowing passes: rank `r` counts from the top of [lo, hi]
    uint32_t r = static_cast<uint32_t>(want);
    uint32_t in_range = static_cast<uint32_t>(n_pool);
    while (lo < hi) {
        const uint32_t width_m1 = hi - lo;                      // >= 1
        const int bits = 32 - __builtin_clz(width_m1);          // width <= 2^bits
        const int shift = bits > kBinsLog2 ? bits - kBinsLog2 : 0;
        for (int b = tid; b < kBins; b += kPlanThreads) sh.hist[b] = 0;
        __syncthreads();
        for (int t = tid; t < T; t += kPlanThreads)
            for (int j = Kb; j < K; ++j) {
                const uint32_t k = ordered_key(topk_s[static_cast<size_t>(t) * K + j]);
                if (k >= lo && k <= hi) atomicAdd(&sh.hist[(k - lo) >> shift], 1u);
            }
        __syncthreads();
        // suffix sums over bins, two adjacent bins per thread, highest bins first:
        // thread i owns bins kBins-1-2i (first) and kBins-2-2i (second)
        const int b_first = kBins - 1 - 2 * tid, b_second = b_first - 1;
        const uint32_t c_first = sh.hist[b_first], c_second = sh.hist[b_second];
        const uint32_t above = block_scan_excl(c_first + c_second, sh.wave_tot, nullptr);
        // `above` = number of in-range keys in bins higher than b_first
        if (above < r && r <= above + c_first) {
            sh.pick_bin = b_first;
            sh.pick_rank = r - above;
            sh.pick_count = c_first;
        } else if (above + c_first < r && r <= above + c_first + c_second) {
            sh.pick_bin = b_second;
            sh.pick_rank = r - above - c_first;
            sh.pick_count = c_second;
        }
        __syncthreads();
        const uint32_t pb = sh.pick_bin;
        r = sh.pick_rank;
        in_range = sh.pick_count;
        const uint32_t new_lo = lo + (pb << shift);
        const uint32_t span_m1 = (shift == 0) ? 0u : ((1u << shift) - 1u);
        const uint32_t new_hi = (hi - new_lo < span_m1) ? hi : new_lo + span_m1;
        lo = new_lo;
        hi = new_hi;
        __syncthreads();
    }
    const uint32_t vstar = lo;      // key of the B'-th largest pool entry
    const uint32_t n_equal = in_range;
    const uint32_t R = r;           // how many of the keys == vstar are kept (1..n_equal)

    if (R == n_equal) {             // no tie is split: a plain threshold
        for (int t = tid; t < T; t += kPlanThreads) {
            int c = Kb;
            for (int j = Kb; j < K; ++j)
                c += ordered_key(topk_s[static_cast<size_t>(t) * K + j]) >= vstar ? 1 : 0;
            keep_count[t] = c;
        }
        return;
    }
    // ---- ties at the threshold: keep the first R equal keys in (token, rank)
    // order.  Tokens are visited in rounds of 1024 (thread = token), so the
    // order is (round, thread, rank); `seen` carries the equal keys of earlier
    // rounds.
    uint32_t seen = 0;
    const int rounds = (T + kPlanThreads - 1) / kPlanThreads;
    for (int it = 0; it < rounds; ++it) {
        const int t = it * kPlanThreads + tid;
        uint32_t gt = 0, eq = 0;
        if (t < T)
            for (int j = Kb; j < K; ++j) {
                const uint32_t k = ordered_key(topk_s[static_cast<size_t>(t) * K + j]);
                gt += k > vstar ? 1u : 0u;
                eq += k == vstar ? 1u : 0u;
            }
        uint32_t round_total;
        const uint32_t before = seen + block_scan_excl(eq, sh.wave_tot, &round_total);
        seen += round_total;
        if (t < T) {
            // equal keys of one token sit at consecutive ranks right after its
            // larger ones, so the first min(eq, R - before) of them are kept
            const uint32_t room = before < R ? R - before : 0u;
            keep_count[t] = Kb + static_cast<int>(gt + min(eq, room));
        }
    }
}

// Rows of the kept pairs in (expert, token) order.  words/prefix: scratch of
// 64 * ceil(T/64) entries each (u64 / i32), indexed [batch * 64 + expert].
__device__ void dispatch_phase(PlanShared& sh, const int32_t* topk_ids,
                               const int32_t* keep_count, int T, int K, int E, int64_t max_rows,
                               int32_t* expert_offsets, int32_t* row_token, int32_t* row_rank,
                               int32_t* inv_row, uint64_t* words, int32_t* prefix) {
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
    const int n_batch = (T + kWave - 1) / kWave;

    // ---- A: per batch, the 64-bit "who keeps expert e" words (lane e owns word e)
    for (int b = wave; b < n_batch; b += kPlanWaves) {
        const int t = b * kWave + lane;
        uint64_t mine = 0;   // bit e: this token keeps expert e
        if (t < T) {
            const int kt = min(K, keep_count[t]);
            for (int j = 0; j < kt; ++j)
                mine |= 1ull << (topk_ids[static_cast<size_t>(t) * K + j] & (kWave - 1));
        }
        uint64_t col = 0;
        for (int e = 0; e < E; ++e) {
            const uint64_t w = __ballot((mine >> e) & 1ull);
            if (lane == e) col = w;
        }
        words[static_cast<size_t>(b) * kWave + lane] = col;
    }
    __threadfence_block();
    __syncthreads();

    // ---- B: per expert, exclusive prefix over batches; then offsets over experts.
    // thread (seg, e): 16 segments of batches per expert.
    {
        const int e = tid % kWave, seg = tid / kWave;
        const int per_seg = (n_batch + kPlanWaves - 1) / kPlanWaves;
        const int b0 = seg * per_seg, b1 = min(n_batch, b0 + per_seg);
        int local = 0;
        for (int b = b0; b < b1; ++b) local += __popcll(words[static_cast<size_t>(b) * kWave + e]);
        sh.hist[seg * kWave + e] = static_cast<uint32_t>(local);
        __syncthreads();
        int base = 0, total = 0;
        for (int s = 0; s < kPlanWaves; ++s) {
            const int v = static_cast<int>(sh.hist[s * kWave + e]);
            if (s < seg) base += v;
            total += v;
        }
        int run = base;
        for (int b = b0; b < b1; ++b) {
            prefix[static_cast<size_t>(b) * kWave + e] = run;
            run += __popcll(words[static_cast<size_t>(b) * kWave + e]);
        }
        if (seg == 0) {
            // wave 0: lane e holds expert e's row count
            const int incl = wave_scan_incl(e < E ? total : 0);
            sh.expert_off[e + 1] = incl;
            if (e == 0) sh.expert_off[0] = 0;
        }
        __threadfence_block();
        __syncthreads();
        // (offsets past the budget can only come from keep counts that sum to more than it)
        if (tid <= E) expert_offsets[tid] = min(sh.expert_off[tid], static_cast<int32_t>(max_rows));
    }

    // ---- C: place every pair
    for (int b = wave; b < n_batch; b += kPlanWaves) {
        const int t = b * kWave + lane;
        if (t >= T) continue;
        const int kt = min(K, keep_count[t]);
        const uint64_t below = lanemask_lt();
        for (int j = 0; j < K; ++j) {
            int row = -1;
            if (j < kt) {
                const int e = topk_ids[static_cast<size_t>(t) * K + j] & (kWave - 1);
                const size_t idx = static_cast<size_t>(b) * kWave + e;
                row = sh.expert_off[e] + prefix[idx] + __popcll(words[idx] & below);
                if (row < max_rows) {   // holds whenever sum_t keep_count[t] <= budget
                    row_token[row] = t;
                    row_rank[row] = j;
                } else {
                    row = -1;           // no row behind this pair: the combine skips it
                }
            }
            inv_row[static_cast<size_t>(t) * K + j] = row;
        }
    }
}

// Tile map of the grouped GEMMs (layout and order: kernels.hpp), written by the
// first wave of the workgroup.  expert_off: the E+1 row offsets (LDS).
__device__ __forceinline__ void write_tile_map(const int32_t* expert_off, int E, int bm,
                                               int32_t* __restrict__ tile_info, int max_rows) {
    const int lane = lane_id();
    // lane = expert: its rows in n tiles of rt rows (the last one may hold fewer); rows past
    // the budget (keep counts that sum to more than it) do not exist
    int off = lane < E ? min(expert_off[lane], max_rows) : 0;
    int rows = lane < E ? min(expert_off[lane + 1], max_rows) - off : 0;
    int n = (rows + bm - 1) / bm;
    int rt = n > 0 ? (rows + n - 1) / n : 0;
    // rank of the expert by (rows per tile descending, expert ascending)
    int rank = 0;
#pragma unroll
    for (int o = 0; o < kWave; ++o) {
        const int ro = __builtin_amdgcn_readlane(rt, o);
        rank += (ro > rt || (ro == rt && o < lane)) ? 1 : 0;
    }
    // from here on lane = rank: fetch the data of the expert with this rank
    int e = 0;
#pragma unroll
    for (int o = 0; o < kWave; ++o) e = __builtin_amdgcn_readlane(rank, o) == lane ? o : e;
    rows = __shfl(rows, e, kWave);
    off = __shfl(off, e, kWave);
    n = __shfl(n, e, kWave);
    rt = __shfl(rt, e, kWave);
    const int incl = wave_scan_incl(n);
    const int first = incl - n;
    for (int i = 0; i < n; ++i) {
        int32_t* ent = tile_info + kTileHdr + 4 * static_cast<size_t>(first + i);
        ent[0] = e;
        ent[1] = off + i * rt;
        ent[2] = min(rt, rows - i * rt);
        ent[3] = n;
    }
    if (lane == kWave - 1) tile_info[0] = incl;
    // [1]: the single tiles of at most 64 rows (they end the list: fewest rows per tile)
    const uint64_t light = __ballot(n == 1 && rt <= 64);
    if (lane == 0) tile_info[1] = __popcll(light);
}

__device__ void tilemap_phase(PlanShared& sh, int E, int bm, int32_t* __restrict__ tile_info,
                              int max_rows) {
    if (threadIdx.x < kWave) write_tile_map(sh.expert_off, E, bm, tile_info, max_rows);
}

// ---------------------------------------------------------------------------
// Fast path (T <= 8192 and at most 48 pool keys per thread): the same two
// phases, but the pool keys are read from global memory once and stay in
// registers for every pass, and the keep counts, ballot words and prefixes live
// in LDS, so no phase waits on a global round trip of its own.
//
// Selection: thread i owns the contiguous slice [i*C, (i+1)*C) of the pool in
// (token, rank) order, so "equal keys that precede" is a block-wide exclusive
// scan of per-thread counts plus a walk through the thread's own keys.
// Dispatch: the 64 x 64 bit matrix "token t of the batch keeps expert e" is
// transposed with a 6-stage butterfly of lane exchanges instead of 64 ballots.
constexpr int kFastMaxT = 8192;
constexpr int kFastMaxKeys = 48;
// Pools up to this size are ranked directly (quadratic in the pool); measured on
// DeepSeek-V2-Lite shapes the histogram search is faster from about 300 entries on
// (T = 64, pool 320: 25 us direct, 17 us by histogram; pool 240: 15 against 18).
constexpr int kDirectPool = 256;
constexpr int kMaxK = 16;          // candidates per token the interface allows

struct FastShared {
    uint32_t hist[kBins];
    uint32_t wave_tot[kPlanWaves];
    uint32_t red_lo[kPlanWaves];
    uint32_t red_hi[kPlanWaves];
    uint32_t pick_bin, pick_rank, pick_count;
    int32_t expert_off[kWave + 1];
    int32_t seg_tot[kPlanWaves][kWave];
    int32_t cnt[kFastMaxT];        // keep_count
    union {
        struct {
            uint64_t words[kFastMaxT];   // [batch][expert]
            int32_t prefix[kFastMaxT];   // [batch][expert]
        };
        // during the selection, before the dispatch arrays are needed: the candidate
        // scores, copied in with coalesced loads
        float stage[kFastMaxT * 3];
    };
};
constexpr int kStageFloats = kFastMaxT * 3;

// Transpose of a 64 x 64 bit matrix held one row per lane: afterwards lane e
// holds column e (bit t = former bit e of lane t).
template <int S>
__device__ __forceinline__ uint64_t transpose_round(uint64_t x, int lane) {
    // bits whose index has bit S clear
    constexpr uint64_t m = S == 32   ? 0x00000000FFFFFFFFull
                           : S == 16 ? 0x0000FFFF0000FFFFull
                           : S == 8  ? 0x00FF00FF00FF00FFull
                           : S == 4  ? 0x0F0F0F0F0F0F0F0Full
                           : S == 2  ? 0x3333333333333333ull
                                     : 0x5555555555555555ull;
    const uint64_t y = lane_xor<S>(x);
    return (lane & S) ? ((x & ~m) | ((y & ~m) >> S)) : ((x & m) | ((y & m) << S));
}
__device__ __forceinline__ uint64_t wave_transpose64(uint64_t x) {
    const int lane = lane_id();
    x = transpose_round<32>(x, lane);
    x = transpose_round<16>(x, lane);
    x = transpose_round<8>(x, lane);
    x = transpose_round<4>(x, lane);
    x = transpose_round<2>(x, lane);
    x = transpose_round<1>(x, lane);
    return x;
}

template <bool SELECT, bool DISPATCH, int NT>
__global__ __launch_bounds__(NT) void plan_fast_kernel(
    const float* topk_s, const int32_t* topk_ids, int T, int K, int Kb, int64_t B, int E,
    int32_t* keep_count, int32_t* expert_offsets, int32_t* row_token, int32_t* row_rank,
    int32_t* inv_row, int bm, int32_t* tile_info) {
    __shared__ FastShared sh;
    constexpr int NW = NT / kWave;            // waves
    constexpr int NBINS = 2 * NT;             // histogram bins: two per thread
    constexpr int NBINS_LOG2 = NT == 1024 ? 11 : 9;
    static_assert(NT == 1024 || NT == 256, "two block sizes");
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
    // Launched as several workgroups (only where nothing else wants the compute units),
    // every workgroup runs the selection and the counting phases redundantly, on its own
    // unit and in its own LDS, with identical results and no exchange between them, and
    // then writes its share of the placement, the one phase that is bound by the number of
    // scattered stores a single compute unit can issue; workgroup 0 writes the rest.
    const int n_groups = gridDim.x, group = blockIdx.x;
    const bool writer = group == 0;

    // Candidate ids of this wave's batches (lane = token), all loaded up front so that
    // the loads are in flight together, and kept in registers for both uses in the
    // dispatch.  The 4-wave kernel (few tokens, one wave per SIMD, registers to spare)
    // issues them before the selection, whose result they do not depend on; the 16-wave
    // kernel after it.  Wider candidate rows than kIdsK fall back to loading them where
    // they are used.
    constexpr int kIdsK = 8;
    constexpr int kMaxBatches = (NT == 1024 ? kFastMaxT : 1024) / kWave / NW;
    const bool ids_held = DISPATCH && K <= kIdsK;
    int held[kMaxBatches][kIdsK];
    auto load_held = [&]() {
        if (!ids_held) return;
#pragma unroll
        for (int bi = 0; bi < kMaxBatches; ++bi) {
            const int t = (wave + bi * NW) * kWave + lane;
#pragma unroll
            for (int j = 0; j < kIdsK; ++j)
                held[bi][j] = (t < T && j < K) ? topk_ids[static_cast<size_t>(t) * K + j] : 0;
        }
    };
    if (NT == 256) load_held();

    if (SELECT) {
        const int P = K - Kb;
        const int n_pool = T * P;
        const int64_t want = B - static_cast<int64_t>(T) * Kb;
        if (want <= 0 || want >= n_pool) {
            const int c = want <= 0 ? Kb : K;
            for (int t = tid; t < T; t += NT) sh.cnt[t] = c;
        } else if (n_pool <= kDirectPool) {
            // Small pool (decode-shaped calls): every pool entry counts the entries that
            // precede it in the order (score descending, token ascending, rank
            // ascending) and is kept iff fewer than B' do.
            // The order as one unsigned number per entry: key, then the complement of the
            // pool index (equal keys: the lower index is the larger number).  A wave keeps
            // 64 entries of the pool at a time in a register pair and broadcasts them one
            // by one through scalar registers, so the inner loop touches no memory.
            static_assert(kDirectPool <= 256 && kDirectPool <= NT, "one entry per thread, 8-bit index");
            for (int t = tid; t < T; t += NT) sh.cnt[t] = Kb;
            for (int i = tid; i < kDirectPool; i += NT)
                sh.hist[i] = i < n_pool
                                 ? ordered_key(topk_s[static_cast<size_t>(i / P) * K + Kb + i % P])
                                 : 0u;   // below every real key (no finite score maps to 0)
            __syncthreads();
            if (wave * kWave < n_pool) {   // uniform per wave
                const uint64_t mine = (static_cast<uint64_t>(sh.hist[tid]) << 8) | (255u - tid);
                int before = 0;
                for (int c = 0; c * kWave < n_pool; ++c) {
                    const int o = c * kWave + lane;
                    const uint64_t theirs = (static_cast<uint64_t>(sh.hist[o]) << 8) | (255u - o);
                    const int lo = static_cast<int>(static_cast<uint32_t>(theirs));
                    const int hi = static_cast<int>(static_cast<uint32_t>(theirs >> 32));
#pragma unroll
                    for (int l = 0; l < kWave; ++l) {
                        const uint64_t other =
                            static_cast<uint32_t>(__builtin_amdgcn_readlane(lo, l)) |
                            (static_cast<uint64_t>(static_cast<uint32_t>(__builtin_amdgcn_readlane(hi, l))) << 32);
                        before += other > mine ? 1 : 0;
                    }
                }
                if (tid < n_pool && before < want) atomicAdd(&sh.cnt[tid / P], 1);   // integer adds: order-free
            }
        } else {
            for (int t = tid; t < T; t += NT) sh.cnt[t] = Kb;
            // ---- this thread's slice of the pool, in (token, rank) order
            const int C = (n_pool + NT - 1) / NT;   // <= kFastMaxKeys
            const int n0 = min(n_pool, tid * C), n_mine = min(n_pool, n0 + C) - n0;
            const int t_first = n0 / P, j_first = n0 % P;
            uint32_t key[kFastMaxKeys];
            // A thread's slice is strided in memory (lane stride = C scores), so where the
            // whole [T,K] score matrix fits the staging area it is copied to LDS with
            // coalesced loads and the slices are read from there.
            const bool staged = T * K <= kStageFloats;
            if (staged) {
                const int n_all = T * K;
                if ((n_all & 3) == 0 && (reinterpret_cast<uintptr_t>(topk_s) & 15) == 0) {
                    const float4* src = reinterpret_cast<const float4*>(topk_s);
                    float4* dst = reinterpret_cast<float4*>(sh.stage);
                    for (int i = tid; i < n_all / 4; i += NT) dst[i] = src[i];
                } else {
                    for (int i = tid; i < n_all; i += NT) sh.stage[i] = topk_s[i];
                }
                __syncthreads();
            }
            {
                int t = t_first, j = j_first;
#pragma unroll
                for (int q = 0; q < kFastMaxKeys; ++q) {
                    key[q] = 0;
                    if (q < n_mine) {
                        const size_t at = static_cast<size_t>(t) * K + Kb + j;
                        key[q] = ordered_key(staged ? sh.stage[at] : topk_s[at]);
                        if (++j == P) { j = 0; ++t; }
                    }
                }
            }
            if (staged) __syncthreads();   // the staging area is the dispatch arrays' from here on
            // ---- range of the keys
            uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
            for (int q = 0; q < kFastMaxKeys; ++q) {
                if (q >= C) continue;
                if (q < n_mine) {
                    lo = min(lo, key[q]);
                    hi = max(hi, key[q]);
                }
            }
            lo = wave_min_u32(lo);
            hi = wave_max_u32(hi);
            if (lane == 0) {
                sh.red_lo[wave] = lo;
                sh.red_hi[wave] = hi;
            }
            if (tid == 0) {
                sh.pick_bin = 0;
                sh.pick_rank = 1;
                sh.pick_count = 1;
            }
            __syncthreads();
            lo = 0xFFFFFFFFu;
            hi = 0u;
            for (int w = 0; w < NW; ++w) {
                lo = min(lo, sh.red_lo[w]);
                hi = max(hi, sh.red_hi[w]);
            }
            // ---- narrowing passes (see select_phase)
            uint32_t r = static_cast<uint32_t>(want);
            uint32_t in_range = static_cast<uint32_t>(n_pool);
            while (lo < hi) {
                const uint32_t width_m1 = hi - lo;
                const int bits = 32 - __builtin_clz(width_m1);
                const int shift = bits > NBINS_LOG2 ? bits - NBINS_LOG2 : 0;
                for (int b = tid; b < NBINS; b += NT) sh.hist[b] = 0;
                __syncthreads();
#pragma unroll
                for (int q = 0; q < kFastMaxKeys; ++q) {
                    if (q >= C) continue;
                    if (q < n_mine && key[q] >= lo && key[q] <= hi)
                        atomicAdd(&sh.hist[(key[q] - lo) >> shift], 1u);
                }
                __syncthreads();
                const int b_first = NBINS - 1 - 2 * tid, b_second = b_first - 1;
                const uint32_t c_first = sh.hist[b_first], c_second = sh.hist[b_second];
                const uint32_t above = block_scan_excl<NW>(c_first + c_second, sh.wave_tot, nullptr);
                if (above < r && r <= above + c_first) {
                    sh.pick_bin = b_first;
                    sh.pick_rank = r - above;
                    sh.pick_count = c_first;
                } else if (above + c_first < r && r <= above + c_first + c_second) {
                    sh.pick_bin = b_second;
                    sh.pick_rank = r - above - c_first;
                    sh.pick_count = c_second;
                }
                __syncthreads();
                const uint32_t pb = sh.pick_bin;
                r = sh.pick_rank;
                in_range = sh.pick_count;
                const uint32_t new_lo = lo + (pb << shift);
                const uint32_t span_m1 = (shift == 0) ? 0u : ((1u << shift) - 1u);
                hi = (hi - new_lo < span_m1) ? hi : new_lo + span_m1;
                lo = new_lo;
                __syncthreads();
            }
            const uint32_t vstar = lo, n_equal = in_range, R = r;
            // ---- equal keys that precede this thread's slice (only if a tie is split)
            uint32_t before = 0;
            if (R != n_equal) {   // uniform
                uint32_t eq = 0;
#pragma unroll
                for (int q = 0; q < kFastMaxKeys; ++q) {
                    if (q >= C) continue;
                    if (q < n_mine) eq += key[q] == vstar ? 1u : 0u;
                }
                before = block_scan_excl<NW>(eq, sh.wave_tot, nullptr);
            }
            // ---- kept entries per token (a token's slice may straddle two threads:
            // integer adds in LDS, order-independent)
            {
                int t = t_first, j = j_first, run = 0;
#pragma unroll
                for (int q = 0; q < kFastMaxKeys; ++q) {
                    if (q >= C) continue;
                    if (q < n_mine) {
                        bool keep = key[q] > vstar;
                        if (key[q] == vstar) {
                            keep = R == n_equal || before < R;
                            ++before;
                        }
                        run += keep ? 1 : 0;
                        if (++j == P || q == n_mine - 1) {
                            if (run) atomicAdd(&sh.cnt[t], run);
                            run = 0;
                            j = 0;
                            ++t;
                        }
                    }
                }
            }
        }
        __syncthreads();
        if (writer)
            for (int t = tid; t < T; t += NT) keep_count[t] = sh.cnt[t];
    } else {
        for (int t = tid; t < T; t += NT) sh.cnt[t] = keep_count[t];
        __syncthreads();
    }
    if (!DISPATCH) return;

    const int n_batch = (T + kWave - 1) / kWave;
    if (NT != 256) load_held();
    // ---- A: ballot words by bit-matrix transpose (lane e ends up with expert e's word)
#pragma unroll
    for (int bi = 0; bi < kMaxBatches; ++bi) {
        const int b = wave + bi * NW;
        if (b >= n_batch) break;
        const int t = b * kWave + lane;
        uint64_t mine = 0;
        if (t < T) {
            const int kt = min(K, sh.cnt[t]);
            if (ids_held) {
#pragma unroll
                for (int j = 0; j < kIdsK; ++j)
                    if (j < kt) mine |= 1ull << (held[bi][j] & (kWave - 1));
            } else {
                int ids[kMaxK];   // all loads first, so that they are in flight together
#pragma unroll
                for (int j = 0; j < kMaxK; ++j)
                    ids[j] = j < K ? topk_ids[static_cast<size_t>(t) * K + j] : 0;
#pragma unroll
                for (int j = 0; j < kMaxK; ++j)
                    if (j < kt) mine |= 1ull << (ids[j] & (kWave - 1));
            }
        }
        sh.words[b * kWave + lane] = wave_transpose64(mine);
    }
    __syncthreads();
    // ---- B: per expert, exclusive prefix over batches; offsets over experts
    {
        const int e = tid % kWave, seg = tid / kWave;
        const int per_seg = (n_batch + NW - 1) / NW;
        const int b0 = min(n_batch, seg * per_seg), b1 = min(n_batch, b0 + per_seg);
        int local = 0;
        for (int b = b0; b < b1; ++b) local += __popcll(sh.words[b * kWave + e]);
        sh.seg_tot[seg][e] = local;
        __syncthreads();
        int base = 0, total = 0;
        for (int s2 = 0; s2 < NW; ++s2) {
            const int v = sh.seg_tot[s2][e];
            if (s2 < seg) base += v;
            total += v;
        }
        int run = base;
        for (int b = b0; b < b1; ++b) {
            sh.prefix[b * kWave + e] = run;
            run += __popcll(sh.words[b * kWave + e]);
        }
        if (seg == 0) {
            const int incl = wave_scan_incl(e < E ? total : 0);
            sh.expert_off[e + 1] = incl;
            if (e == 0) sh.expert_off[0] = 0;
        }
        __syncthreads();
        if (writer && tid <= E) expert_offsets[tid] = min(sh.expert_off[tid], static_cast<int32_t>(B));
    }
    // ---- tile map, by the last wave, beside the other waves' share of phase C (with few
    // tokens the last wave has no batch of its own)
    if (writer && tile_info != nullptr && wave == NW - 1)
        write_tile_map(sh.expert_off, E, bm, tile_info, static_cast<int>(B));
    // ---- C: place every pair (token t = lane of batch b, candidate ids in `ids`)
    auto place = [&](int b, int t, const int (&ids)[kMaxK]) {
        const int kt = min(K, sh.cnt[t]);
        const uint64_t below = lanemask_lt();
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) {
            if (j >= K) continue;
            int row = -1;
            if (j < kt) {
                const int e = ids[j] & (kWave - 1);
                const int idx = b * kWave + e;
                row = sh.expert_off[e] + sh.prefix[idx] + __popcll(sh.words[idx] & below);
                if (row < B) {   // holds whenever sum_t keep_count[t] <= budget
                    row_token[row] = t;
                    row_rank[row] = j;
                } else {
                    row = -1;
                }
            }
            inv_row[static_cast<size_t>(t) * K + j] = row;
        }
    };
    if (n_groups == 1) {
#pragma unroll
        for (int bi = 0; bi < kMaxBatches; ++bi) {
            const int b = wave + bi * NW;
            if (b >= n_batch) break;
            const int t = b * kWave + lane;
            if (t >= T) continue;
            int ids[kMaxK];
#pragma unroll
            for (int j = 0; j < kMaxK; ++j) {
                if (ids_held)
                    ids[j] = j < kIdsK ? held[bi][j < kIdsK ? j : 0] : 0;
                else
                    ids[j] = j < K ? topk_ids[static_cast<size_t>(t) * K + j] : 0;
            }
            place(b, t, ids);
        }
    } else {
        // several workgroups: each has computed the same counts, words and prefixes and
        // places the batches group, group + n_groups, ..., one per wave at a time
        for (int b = group + n_groups * wave; b < n_batch; b += n_groups * NW) {
            const int t = b * kWave + lane;
            if (t >= T) continue;
            int ids[kMaxK];
#pragma unroll
            for (int j = 0; j < kMaxK; ++j)
                ids[j] = j < K ? topk_ids[static_cast<size_t>(t) * K + j] : 0;
            place(b, t, ids);
        }
    }
}

// ---------------------------------------------------------------------------
// Many tokens (T >= kPlanSpreadTokens): the same selection and dispatch spread over
// workgroups, as a fixed sequence of short launches, with no global atomics and no
// waiting between workgroups (what a later launch needs from all workgroups of an
// earlier one goes through memory).
//
// Selection: exact radix select of the B'-th largest pool key on the 32 key bits, 11 +
// 11 + 10 from the top.  Pass p: each of G workgroups histograms, in LDS, the digit p of
// its share of the pool keys whose higher digits equal the ones already found, and writes
// its 2048 counts to hist[p][g]; the next launch sums the G partial histograms per bin,
// walks them from the top and finds the digit that holds the wanted rank (every workgroup
// does this redundantly, workgroup 0 records digit and remaining rank for the launches
// after it).  After three passes the key v* and the number R of keys equal to v* that
// are kept are known.  keep: thread = token; ties at v* are split in (token, rank) order:
// a workgroup counts the equal keys of all earlier tokens itself (only when a tie is
// split).  The same launch forms the ballot words of its batches of 64 tokens.
// place: a workgroup owns 16 batches; per expert (lane) the counts of all batches and of
// the batches before its own come from popcounts of the ballot words; then the rows.
constexpr int kSpreadThreads = 1024;   // (kPlanSpreadTokens: kernels.hpp)
constexpr int kSpreadMaxGroups = 16;
constexpr int kSpreadBins = 2048;

struct SpreadState {
    uint32_t b1, r1, b2, r2;
};

inline int spread_groups(int T) {
    const int g = (T + kSpreadThreads - 1) / kSpreadThreads;
    return g < kSpreadMaxGroups ? g : kSpreadMaxGroups;
}

size_t plan_spread_bytes(int T) {
    if (T < kPlanSpreadTokens) return 0;
    return 3 * static_cast<size_t>(spread_groups(T)) * kSpreadBins * sizeof(uint32_t) + 256;
}

// The bin (of the G partial histograms summed) that holds the r-th largest key counted
// from the top bin, the rank inside it and its count.  Block-wide; every thread returns
// the same values.
__device__ __forceinline__ void spread_find_bin(const uint32_t* __restrict__ partials, int G,
                                                uint32_t r, uint32_t* wave_tot, uint32_t* pick,
                                                uint32_t& bin, uint32_t& rank, uint32_t& count) {
    const int tid = threadIdx.x;
    const int b_first = kSpreadBins - 1 - 2 * tid, b_second = b_first - 1;
    uint32_t c_first = 0, c_second = 0;
    for (int g = 0; g < G; ++g) {
        c_first += partials[static_cast<size_t>(g) * kSpreadBins + b_first];
        c_second += partials[static_cast<size_t>(g) * kSpreadBins + b_second];
    }
    const uint32_t above = block_scan_excl(c_first + c_second, wave_tot, nullptr);
    if (above < r && r <= above + c_first) {
        pick[0] = b_first;
        pick[1] = r - above;
        pick[2] = c_first;
    } else if (above + c_first < r && r <= above + c_first + c_second) {
        pick[0] = b_second;
        pick[1] = r - above - c_first;
        pick[2] = c_second;
    }
    __syncthreads();
    bin = pick[0];
    rank = pick[1];
    count = pick[2];
    __syncthreads();
}

template <int PASS>
__global__ __launch_bounds__(kSpreadThreads) void spread_hist_kernel(
    const float* __restrict__ keys, int T, int K, int Kb, int64_t B, uint32_t* __restrict__ hist,
    int G, SpreadState* __restrict__ state) {
    __shared__ uint32_t h[kSpreadBins];
    __shared__ uint32_t wave_tot[kPlanWaves];
    __shared__ uint32_t pick[3];
    const int tid = threadIdx.x;
    const int P = K - Kb;
    const int64_t n_pool = static_cast<int64_t>(T) * P, want = B - static_cast<int64_t>(T) * Kb;
    if (want <= 0 || want >= n_pool) return;   // nothing or everything from the pool: no search
    uint32_t b1 = 0, b2 = 0;
    if (PASS == 2) {
        uint32_t r1, c;
        spread_find_bin(hist, G, static_cast<uint32_t>(want), wave_tot, pick, b1, r1, c);
        if (blockIdx.x == 0 && tid == 0) {
            state->b1 = b1;
            state->r1 = r1;
        }
    } else if (PASS == 3) {
        b1 = state->b1;
        uint32_t r2, c;
        spread_find_bin(hist + static_cast<size_t>(G) * kSpreadBins, G, state->r1, wave_tot, pick, b2,
                        r2, c);
        if (blockIdx.x == 0 && tid == 0) {
            state->b2 = b2;
            state->r2 = r2;
        }
    }
    for (int b = tid; b < kSpreadBins; b += kSpreadThreads) h[b] = 0;
    __syncthreads();
    const int per = (T + G - 1) / G;
    const int t_begin = blockIdx.x * per, t_end = min(T, t_begin + per);
    for (int t = t_begin + tid; t < t_end; t += kSpreadThreads)
        for (int j = Kb; j < K; ++j) {
            const uint32_t k = ordered_key(keys[static_cast<size_t>(t) * K + j]);
            if (PASS == 1)
                atomicAdd(&h[k >> 21], 1u);
            else if (PASS == 2) {
                if ((k >> 21) == b1) atomicAdd(&h[(k >> 10) & 0x7FFu], 1u);
            } else {
                if ((k >> 10) == ((b1 << 11) | b2)) atomicAdd(&h[k & 0x3FFu], 1u);
            }
        }
    __syncthreads();
    uint32_t* out = hist + (static_cast<size_t>(PASS - 1) * G + blockIdx.x) * kSpreadBins;
    for (int b = tid; b < kSpreadBins; b += kSpreadThreads) out[b] = h[b];
}

// keep_count of the workgroup's 1024 tokens (SELECT; otherwise they are read) and the ballot
// words of its 16 batches (words may be null: selection only).
template <bool SELECT>
__global__ __launch_bounds__(kSpreadThreads) void spread_keep_kernel(
    const float* __restrict__ keys, const int32_t* __restrict__ topk_ids, int T, int K, int Kb,
    int64_t B, const uint32_t* __restrict__ hist, int G, const SpreadState* __restrict__ state,
    int32_t* __restrict__ keep_count, uint64_t* __restrict__ words) {
    __shared__ uint32_t wave_tot[kPlanWaves];
    __shared__ uint32_t pick[3];
    const int tid = threadIdx.x, lane = lane_id();
    const int t0 = blockIdx.x * kSpreadThreads, t = t0 + tid;
    int keep = 0;
    if (SELECT) {
        const int P = K - Kb;
        const int64_t n_pool = static_cast<int64_t>(T) * P, want = B - static_cast<int64_t>(T) * Kb;
        if (want <= 0 || want >= n_pool) {
            keep = want <= 0 ? Kb : K;
        } else {
            uint32_t b3, R, n_equal;
            spread_find_bin(hist + 2 * static_cast<size_t>(G) * kSpreadBins, G, state->r2, wave_tot,
                            pick, b3, R, n_equal);
            const uint32_t vstar = (state->b1 << 21) | (state->b2 << 10) | b3;
            uint32_t gt = 0, eq = 0;
            if (t < T)
                for (int j = Kb; j < K; ++j) {
                    const uint32_t k = ordered_key(keys[static_cast<size_t>(t) * K + j]);
                    gt += k > vstar ? 1u : 0u;
                    eq += k == vstar ? 1u : 0u;
                }
            if (R == n_equal) {   // no tie is split: a plain threshold
                keep = Kb + static_cast<int>(gt + eq);
            } else {
                // equal keys of the tokens before this workgroup's, counted here
                uint32_t mine = 0;
                for (int u = tid; u < t0; u += kSpreadThreads)
                    for (int j = Kb; j < K; ++j)
                        mine += ordered_key(keys[static_cast<size_t>(u) * K + j]) == vstar ? 1u : 0u;
                uint32_t earlier;
                block_scan_excl(mine, wave_tot, &earlier);
                const uint32_t before = earlier + block_scan_excl(eq, wave_tot, nullptr);
                // a token's equal keys sit at consecutive ranks right after its larger ones
                const uint32_t room = before < R ? R - before : 0u;
                keep = Kb + static_cast<int>(gt + min(eq, room));
            }
        }
        if (t < T) keep_count[t] = keep;
    } else if (t < T) {
        keep = keep_count[t];
    }
    if (words == nullptr) return;
    uint64_t mine = 0;   // bit e: this token keeps expert e
    if (t < T) {
        const int kt = min(K, keep);
        int ids[kMaxK];   // all loads first, so that they are in flight together
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) ids[j] = j < K ? topk_ids[static_cast<size_t>(t) * K + j] : 0;
#pragma unroll
        for (int j = 0; j < kMaxK; ++j)
            if (j < kt) mine |= 1ull << (ids[j] & (kWave - 1));
    }
    const uint64_t col = wave_transpose64(mine);   // lane e: who of the batch keeps expert e
    if (t0 + (tid / kWave) * kWave < T) words[static_cast<size_t>(t / kWave) * kWave + lane] = col;
}

__global__ __launch_bounds__(kSpreadThreads) void spread_place_kernel(
    const int32_t* __restrict__ topk_ids, const int32_t* __restrict__ keep_count, int T, int K,
    int E, int64_t B, const uint64_t* __restrict__ words, int32_t* __restrict__ expert_offsets,
    int32_t* __restrict__ row_token, int32_t* __restrict__ row_rank, int32_t* __restrict__ inv_row,
    int bm, int32_t* __restrict__ tile_info) {
    __shared__ int32_t part_before[kPlanWaves][kWave];
    __shared__ int32_t part_total[kPlanWaves][kWave];
    __shared__ int32_t expert_off[kWave + 1];
    __shared__ int32_t before[kWave];
    __shared__ uint64_t wd[kPlanWaves][kWave];
    __shared__ int32_t pre[kPlanWaves][kWave];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
    const int n_batch = (T + kWave - 1) / kWave;
    const int b0 = blockIdx.x * kPlanWaves;
    {   // lane = expert; the waves split the batches
        const int per_seg = (n_batch + kPlanWaves - 1) / kPlanWaves;
        const int s0 = min(n_batch, wave * per_seg), s1 = min(n_batch, s0 + per_seg);
        int tot = 0, bef = 0;
        for (int b = s0; b < s1; ++b) {
            const int c = __popcll(words[static_cast<size_t>(b) * kWave + lane]);
            tot += c;
            bef += b < b0 ? c : 0;
        }
        part_total[wave][lane] = tot;
        part_before[wave][lane] = bef;
    }
    __syncthreads();
    if (wave == 0) {
        int tot = 0, bef = 0;
        for (int w = 0; w < kPlanWaves; ++w) {
            tot += part_total[w][lane];
            bef += part_before[w][lane];
        }
        const int incl = wave_scan_incl(lane < E ? tot : 0);
        expert_off[lane + 1] = incl;
        if (lane == 0) expert_off[0] = 0;
        before[lane] = bef;
    }
    __syncthreads();
    if (blockIdx.x == 0) {
        if (tid <= E) expert_offsets[tid] = min(expert_off[tid], static_cast<int32_t>(B));
        if (tile_info != nullptr && wave == kPlanWaves - 1)
            write_tile_map(expert_off, E, bm, tile_info, static_cast<int>(B));
    }
    const int b = b0 + wave;
    if (b < n_batch) {
        int p = before[lane];
        for (int bb = b0; bb < b; ++bb) p += __popcll(words[static_cast<size_t>(bb) * kWave + lane]);
        pre[wave][lane] = p;
        wd[wave][lane] = words[static_cast<size_t>(b) * kWave + lane];
    }
    __syncthreads();
    const int t = b * kWave + lane;
    if (b >= n_batch || t >= T) return;
    const int kt = min(K, keep_count[t]);
    const uint64_t below = lanemask_lt();
    int ids[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) ids[j] = j < K ? topk_ids[static_cast<size_t>(t) * K + j] : 0;
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
        if (j >= K) continue;
        int row = -1;
        if (j < kt) {
            const int e = ids[j] & (kWave - 1);
            row = expert_off[e] + pre[wave][e] + __popcll(wd[wave][e] & below);
            if (row < B) {   // holds whenever sum_t keep_count[t] <= budget
                row_token[row] = t;
                row_rank[row] = j;
            } else {
                row = -1;
            }
        }
        inv_row[static_cast<size_t>(t) * K + j] = row;
    }
}

// the launches of the spread selection (hist: plan_spread_bytes(T) bytes of scratch)
static void launch_spread_select(const float* keys, const int32_t* topk_ids, int T, int K, int Kb,
                                 int64_t B, void* spread, int32_t* keep_count, uint64_t* words,
                                 hipStream_t stream) {
    const int G = spread_groups(T);
    uint32_t* hist = static_cast<uint32_t*>(spread);
    SpreadState* state = reinterpret_cast<SpreadState*>(hist + 3 * static_cast<size_t>(G) * kSpreadBins);
    const dim3 block(kSpreadThreads);
    hipLaunchKernelGGL(spread_hist_kernel<1>, dim3(G), block, 0, stream, keys, T, K, Kb, B, hist, G, state);
    hipLaunchKernelGGL(spread_hist_kernel<2>, dim3(G), block, 0, stream, keys, T, K, Kb, B, hist, G, state);
    hipLaunchKernelGGL(spread_hist_kernel<3>, dim3(G), block, 0, stream, keys, T, K, Kb, B, hist, G, state);
    hipLaunchKernelGGL(spread_keep_kernel<true>, dim3((T + kSpreadThreads - 1) / kSpreadThreads), block,
                       0, stream, keys, topk_ids, T, K, Kb, B, hist, G, state, keep_count, words);
}

// 0: large sizes (generic kernels), 256 / 1024: block size of the fast kernel.
// Small problems run on 4 waves (one per SIMD): the kernel is a chain of short
// dependent phases, and fewer waves means each instruction issues sooner.
inline int fast_path_threads(int T, int K, int Kb) {
    const int64_t n_pool = static_cast<int64_t>(T) * (K - Kb);
    if (T > kFastMaxT) return 0;
    if (T <= 1024 && (n_pool + 255) / 256 <= kFastMaxKeys) return 256;
    return (n_pool + kPlanThreads - 1) / kPlanThreads <= kFastMaxKeys ? kPlanThreads : 0;
}

// Workgroups of the fast kernel's launch: one beside other work (more would queue behind
// it); alone on the chip as many as leave two 64-token batches of placement to each.
inline int fast_path_groups(int T, bool alone) {
    if (!alone) return 1;
    const int n_batch = (T + kWave - 1) / kWave;
    return std::max(1, std::min(16, n_batch / 2));
}

__global__ __launch_bounds__(kPlanThreads) void select_kernel(const float* topk_s, int T, int K,
                                                              int Kb, int64_t B,
                                                              int32_t* keep_count) {
    __shared__ PlanShared sh;
    select_phase(sh, topk_s, T, K, Kb, B, keep_count);
}

__global__ __launch_bounds__(kPlanThreads) void dispatch_kernel(
    const int32_t* topk_ids, const int32_t* keep_count, int T, int K, int E, int64_t B,
    int32_t* expert_offsets, int32_t* row_token, int32_t* row_rank, int32_t* inv_row,
    uint64_t* words, int32_t* prefix, int bm, int32_t* tile_info) {
    __shared__ PlanShared sh;
    dispatch_phase(sh, topk_ids, keep_count, T, K, E, B, expert_offsets, row_token, row_rank,
                   inv_row, words, prefix);
    if (tile_info != nullptr) tilemap_phase(sh, E, bm, tile_info, static_cast<int>(B));
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(
    const float* topk_s, const int32_t* topk_ids, int T, int K, int Kb, int64_t B, int E,
    int32_t* keep_count, int32_t* expert_offsets, int32_t* row_token, int32_t* row_rank,
    int32_t* inv_row, uint64_t* words, int32_t* prefix, int bm, int32_t* tile_info) {
    __shared__ PlanShared sh;
    select_phase(sh, topk_s, T, K, Kb, B, keep_count);
    __threadfence_block();
    __syncthreads();
    dispatch_phase(sh, topk_ids, keep_count, T, K, E, B, expert_offsets, row_token, row_rank,
                   inv_row, words, prefix);
    if (tile_info != nullptr) tilemap_phase(sh, E, bm, tile_info, static_cast<int>(B));
}

// Keys of the calibrated baseline selectors (include/allocmoe.h, allocmoe_selector),
// one thread per token, fp32: mode 1 -> minus the score mass before candidate j
// (sequential adds), mode 2 -> s[t,j] / s[t,0] (correctly rounded division).
__global__ __launch_bounds__(256) void selector_keys_kernel(const float* __restrict__ topk_s, int T,
                                                            int K, int mode,
                                                            float* __restrict__ keys) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const float* s = topk_s + static_cast<size_t>(t) * K;
    float* k = keys + static_cast<size_t>(t) * K;
    if (mode == 1) {
        float mass = 0.f;
        for (int j = 0; j < K; ++j) {
            k[j] = -mass;
            mass = __fadd_rn(mass, s[j]);
        }
    } else {
        const float top = s[0];
        for (int j = 0; j < K; ++j) k[j] = top > 0.f ? __fdiv_rn(s[j], top) : 0.f;
    }
}

hipError_t launch_selector_keys(const float* topk_s, int T, int K, int mode, float* keys,
                                hipStream_t stream) {
    hipLaunchKernelGGL(selector_keys_kernel, dim3((T + 255) / 256), dim3(256), 0, stream, topk_s, T,
                       K, mode, keys);
    return hipGetLastError();
}

hipError_t launch_select(const float* topk_s, int T, int K, int Kb, int64_t B,
                         int32_t* keep_count, void* spread, hipStream_t stream) {
    if (spread != nullptr && T >= kPlanSpreadTokens) {
        launch_spread_select(topk_s, nullptr, T, K, Kb, B, spread, keep_count, nullptr, stream);
        return hipGetLastError();
    }
    const int nt = fast_path_threads(T, K, Kb);
    if (nt == 256)
        hipLaunchKernelGGL((plan_fast_kernel<true, false, 256>), dim3(1), dim3(256), 0, stream,
                           topk_s, nullptr, T, K, Kb, B, 0, keep_count, nullptr, nullptr, nullptr,
                           nullptr, 0, nullptr);
    else if (nt == 1024)
        hipLaunchKernelGGL((plan_fast_kernel<true, false, 1024>), dim3(1), dim3(1024), 0, stream,
                           topk_s, nullptr, T, K, Kb, B, 0, keep_count, nullptr, nullptr, nullptr,
                           nullptr, 0, nullptr);
    else
        hipLaunchKernelGGL(select_kernel, dim3(1), dim3(kPlanThreads), 0, stream, topk_s, T, K, Kb,
                           B, keep_count);
    return hipGetLastError();
}

hipError_t launch_dispatch(const int32_t* topk_ids, const int32_t* keep_count, int T, int K,
                           int E, int64_t B, int32_t* expert_offsets, int32_t* row_token,
                           int32_t* row_rank, int32_t* inv_row, uint64_t* words, int32_t* prefix,
                           int bm, int32_t* tile_info, bool alone, hipStream_t stream) {
    if (T >= kPlanSpreadTokens) {
        const dim3 grid((T + kSpreadThreads - 1) / kSpreadThreads), block(kSpreadThreads);
        hipLaunchKernelGGL(spread_keep_kernel<false>, grid, block, 0, stream, nullptr, topk_ids, T, K,
                           0, B, nullptr, 0, nullptr, const_cast<int32_t*>(keep_count), words);
        hipLaunchKernelGGL(spread_place_kernel, grid, block, 0, stream, topk_ids, keep_count, T, K, E,
                           B, words, expert_offsets, row_token, row_rank, inv_row, bm, tile_info);
        return hipGetLastError();
    }
    const int nt = fast_path_threads(T, K, K);
    const dim3 groups(fast_path_groups(T, alone));
    if (nt == 256)
        hipLaunchKernelGGL((plan_fast_kernel<false, true, 256>), groups, dim3(256), 0, stream,
                           nullptr, topk_ids, T, K, 0, B, E, const_cast<int32_t*>(keep_count),
                           expert_offsets, row_token, row_rank, inv_row, bm, tile_info);
    else if (nt == 1024)
        hipLaunchKernelGGL((plan_fast_kernel<false, true, 1024>), groups, dim3(1024), 0, stream,
                           nullptr, topk_ids, T, K, 0, B, E, const_cast<int32_t*>(keep_count),
                           expert_offsets, row_token, row_rank, inv_row, bm, tile_info);
    else
        hipLaunchKernelGGL(dispatch_kernel, dim3(1), dim3(kPlanThreads), 0, stream, topk_ids,
                           keep_count, T, K, E, B, expert_offsets, row_token, row_rank, inv_row,
                           words, prefix, bm, tile_info);
    return hipGetLastError();
}

hipError_t launch_plan(const float* topk_s, const int32_t* topk_ids, int T, int K, int Kb,
                       int64_t B, int E, int32_t* keep_count, int32_t* expert_offsets,
                       int32_t* row_token, int32_t* row_rank, int32_t* inv_row, uint64_t* words,
                       int32_t* prefix, int bm, int32_t* tile_info, void* spread, bool alone,
                       hipStream_t stream) {
    if (spread != nullptr && T >= kPlanSpreadTokens) {
        launch_spread_select(topk_s, topk_ids, T, K, Kb, B, spread, keep_count, words, stream);
        const dim3 grid((T + kSpreadThreads - 1) / kSpreadThreads), block(kSpreadThreads);
        hipLaunchKernelGGL(spread_place_kernel, grid, block, 0, stream, topk_ids, keep_count, T, K, E,
                           B, words, expert_offsets, row_token, row_rank, inv_row, bm, tile_info);
        return hipGetLastError();
    }
    const int nt = fast_path_threads(T, K, Kb);
    const dim3 groups(fast_path_groups(T, alone));
    if (nt == 256)
        hipLaunchKernelGGL((plan_fast_kernel<true, true, 256>), groups, dim3(256), 0, stream,
                           topk_s, topk_ids, T, K, Kb, B, E, keep_count, expert_offsets, row_token,
                           row_rank, inv_row, bm, tile_info);
    else if (nt == 1024)
        hipLaunchKernelGGL((plan_fast_kernel<true, true, 1024>), groups, dim3(1024), 0, stream,
                           topk_s, topk_ids, T, K, Kb, B, E, keep_count, expert_offsets, row_token,
                           row_rank, inv_row, bm, tile_info);
    else
        hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, stream, topk_s, topk_ids,
                           T, K, Kb, B, E, keep_count, expert_offsets, row_token, row_rank,
                           inv_row, words, prefix, bm, tile_info);
    return hipGetLastError();
}

}  // namespace allocmoe
