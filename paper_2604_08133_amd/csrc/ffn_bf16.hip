// bf16 expert networks on the matrix cores (Section 3.1: one feed-forward
// execution per selected pair), fp32 accumulation, from weights re-tiled once
// into MFMA fragment order (pack.hip):
//   H = silu(A W1) * (A W3)   (SWIGLU, bf16 out)    or    O = A W2   (fp32 out).
//
// Weight-streaming kernel.  For token counts where an expert sees only a few
// rows the layer is bound by reading each active expert's weights once from
// HBM.  A workgroup owns one (row tile of <= 32 rows, block of 32 output
// columns); its 4 waves split the contraction dimension, each streaming its
// slice of the packed weight fragments straight from global memory into MFMA B
// operands (1 KB contiguous per wave-load, every byte read once), with many
// independent loads in flight.  The A operand (<= 32 activation rows, L2
// resident) is gathered per lane.  Partial accumulators meet in LDS in a fixed
// order, so results are bitwise reproducible.
#include "common.hpp"
#include "kernels.hpp"

namespace allocmoe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kStreamWaves = 4;
constexpr int kStreamUnroll = 8;

// 32x32 accumulator layout of v_mfma_f32_32x32x16_bf16: register r of lane l
// holds C[8*(r/4) + 4*(l/32) + r%4][l%32].
__device__ __forceinline__ int acc_row(int r, int l) { return 8 * (r / 4) + 4 * (l / 32) + (r % 4); }

template <bool SWIGLU>
__global__ __launch_bounds__(kStreamWaves* kWave) void ffn_bf16_stream_kernel(StreamGroup g0,
                                                                             StreamGroup g1) {
    constexpr int NACC = SWIGLU ? 2 : 1;
    __shared__ float red[kStreamWaves][NACC][16][kWave];

    // the grid is the routed group's workgroups followed by the shared expert's
    const bool first = static_cast<int64_t>(blockIdx.x) < g0.n_wg;
    const StreamGroup& g = first ? g0 : g1;
    const int bid = first ? blockIdx.x : blockIdx.x - static_cast<unsigned>(g0.n_wg);
    const bf16_t* __restrict__ A = static_cast<const bf16_t*>(g.A);
    const bf16_t* __restrict__ Bp = static_cast<const bf16_t*>(g.Bp);
    const int32_t* __restrict__ row_map = g.row_map;
    const int32_t* __restrict__ tile_info = g.tile_info;
    const int lda = g.lda, Kd = g.Kd, N = g.N, ldc = g.ldc, M_dense = g.M_dense;
    const size_t group_stride = g.group_stride;
    void* Cv = g.C;

    const int n_blocks = N / 32;
    const int tile = bid / n_blocks, nb = bid % n_blocks;
    int e, row0, rows;
    if (tile_info != nullptr) {
        if (tile >= tile_info[0]) return;
        const int32_t* ent = tile_info + 4 + 4 * static_cast<size_t>(tile);
        e = ent[0];
        row0 = ent[1];
        rows = ent[2];
    } else {
        e = 0;
        row0 = tile * 32;
        if (row0 >= M_dense) return;
        rows = min(32, M_dense - row0);
    }
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int KB = Kd / 16;                 // k16 steps in total
    const int steps = KB / kStreamWaves;    // per wave (Kd is a multiple of 64)
    const int kb0 = wave * steps;

    // packed B: for this expert and column block, KB fragments of 64 x bf16x8
    // (W1 stream, then for SWIGLU the W3 stream)
    const bf16x8* b1 = reinterpret_cast<const bf16x8*>(
                           Bp + static_cast<size_t>(e) * group_stride +
                           static_cast<size_t>(nb) * (static_cast<size_t>(NACC) * Kd * 32)) +
                       static_cast<size_t>(kb0) * kWave + lane;
    const bf16x8* b3 = b1 + static_cast<size_t>(KB) * kWave;

    // A: lane (m = l%32, kg = l/32) reads 8 consecutive k of its row per step
    const int m = lane % 32, kg = lane / 32;
    const bool a_ok = m < rows;
    long src = 0;
    if (a_ok) {
        const int r = row0 + m;
        src = row_map ? row_map[r] : r;
    }
    const bf16x8* ap =
        reinterpret_cast<const bf16x8*>(A + static_cast<size_t>(src) * lda) + kb0 * 2 + kg;

    f32x16 acc1 = {0}, acc3 = {0};
    const bf16x8 zero = {0};
    int s = 0;
    for (; s + kStreamUnroll <= steps; s += kStreamUnroll) {
        bf16x8 av[kStreamUnroll], w1[kStreamUnroll], w3[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            w1[u] = __builtin_nontemporal_load(b1 + static_cast<size_t>(s + u) * kWave);
            if (SWIGLU) w3[u] = __builtin_nontemporal_load(b3 + static_cast<size_t>(s + u) * kWave);
            av[u] = a_ok ? ap[(s + u) * 2] : zero;
        }
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[u], w1[u], acc1, 0, 0, 0);
            if (SWIGLU) acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[u], w3[u], acc3, 0, 0, 0);
        }
    }
    for (; s < steps; ++s) {
        const bf16x8 w1 = __builtin_nontemporal_load(b1 + static_cast<size_t>(s) * kWave);
        const bf16x8 av = a_ok ? ap[s * 2] : zero;
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, w1, acc1, 0, 0, 0);
        if (SWIGLU) {
            const bf16x8 w3 = __builtin_nontemporal_load(b3 + static_cast<size_t>(s) * kWave);
            acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, w3, acc3, 0, 0, 0);
        }
    }

#pragma unroll
    for (int r = 0; r < 16; ++r) {
        red[wave][0][r][lane] = acc1[r];
        if (SWIGLU) red[wave][NACC - 1][r][lane] = acc3[r];
    }
    __syncthreads();
    // 16 x 64 accumulator slots, 256 threads: 4 slots each, waves summed in order
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int slot = threadIdx.x + 256 * q, r = slot / kWave, l = slot % kWave;
        float v1 = 0.f, v3 = 0.f;
#pragma unroll
        for (int w = 0; w < kStreamWaves; ++w) {
            v1 += red[w][0][r][l];
            if (SWIGLU) v3 += red[w][NACC - 1][r][l];
        }
        const int mr = acc_row(r, l), n = nb * 32 + (l % 32);
        if (mr < rows) {
            const size_t off = static_cast<size_t>(row0 + mr) * ldc + n;
            if (SWIGLU)
                static_cast<bf16_t*>(Cv)[off] = f32_to_bf16((v1 / (1.f + __expf(-v1))) * v3);
            else
                static_cast<float*>(Cv)[off] = v1;
        }
    }
}

// ---------------------------------------------------------------------------
// Tiled kernel for prefill-shaped layers (tens to thousands of rows per expert).
//
// A workgroup of 8 waves owns a tile of <= 256 rows of one expert times 128
// SwiGLU columns (128 of W1 and the same 128 of W3; for the second GEMM: 256
// columns of W2), i.e. 256 x 256 accumulators: per contraction step the
// workgroup pulls (256 + 256) x 32 operands for 2*256*256*32 flop, which keeps
// the L1/LDS fill rate at about half of what the matrix cores could consume.
// Wave (wm, wn): column block wn (32 W1-columns + 32 W3-columns, or 2 x 32
// W2-columns) times the row blocks wm, wm+2, wm+4, wm+6 of 32 rows -- interleaved
// so that a partly filled tile still splits evenly over the two wave rows; row
// blocks without real rows are skipped.  4 x 2 MFMA accumulators of 32x32 per
// wave.  The contraction runs in steps of 32 through a 4-stage LDS ring filled
// by direct-to-LDS loads (16 B per lane, 1 KB per wave-load, no VGPR staging):
// A fragments are gathered row by row straight into MFMA operand order, the
// re-tiled weights are already in that order, so every fragment is read back
// with one conflict-free ds_read_b128.  Loads of steps kt+1..kt+3 are in flight
// while step kt is multiplied; one barrier per step.
constexpr int kTiledRows = 256;
constexpr int kTiledK = 32;
constexpr int kTiledStages = 4;         // 3 is ~13% slower, 5 (all 160 KB of LDS) no faster
constexpr int kTiledWaves = 8;
constexpr int kXcds = 8;                // accelerator dies (one L2 each) of an MI355X
constexpr int kTiledLoadsPerStep = 4;   // per wave: 2 A fragments + 2 B fragments

struct alignas(16) TiledStage {
    bf16x8 a[8][2][kWave];      // [row block][16-row half][position], see the kernel
    bf16x8 b[4][2][2][kWave];   // [column block][stream][k16 half][lane]
};

__device__ __forceinline__ void load_to_lds(const bf16x8* gptr, bf16x8* lds_frag) {
    // lane l's 16 bytes land at lds_frag + l (the hardware adds lane * 16 to the base).
    // Default cache policy: marking the weight stream non-temporal measured ~8% slower.
    __builtin_amdgcn_global_load_lds(gptr, reinterpret_cast<__attribute__((address_space(3))) void*>(
                                               reinterpret_cast<uintptr_t>(lds_frag)),
                                     16, 0, 0);
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence
// would wait for every outstanding direct-to-LDS load, i.e. also for the
// prefetched steps.  The loads a step needs are awaited explicitly (vmcnt)
// before the barrier; the empty asm statements keep the compiler from moving
// LDS accesses across it.
__device__ __forceinline__ void wg_barrier_nofence() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int N>
__device__ __forceinline__ void wait_lgkmcnt_le() {
    // LDS reads return in order: "at most N outstanding" = all but the newest N landed
    __builtin_amdgcn_s_waitcnt(0xC07F | ((N & 15) << 8));
}

template <int N>
__device__ __forceinline__ void wait_vmcnt_le() {
    // s_waitcnt with expcnt/lgkmcnt unconstrained; vmcnt is bits [3:0] and [15:14]
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Main loop and epilogue for a wave that owns NRB row blocks with real rows.
template <bool SWIGLU, int NRB>
__device__ __forceinline__ void tiled_body(TiledStage* st, const bf16x8* ap0, const bf16x8* ap1,
                                           const bf16x8* bsrc,
                                           int KT, int wm, int wn, int lane, int row0, int rows,
                                           int nt, void* C, int ldc) {
    const int wave = wm * 4 + wn;
    auto issue = [&](int kt, int stage) {
        TiledStage& S = st[stage];
        load_to_lds(ap0 + kt * 4, &S.a[wave][0][0]);
        load_to_lds(ap1 + kt * 4, &S.a[wave][1][0]);
        const size_t f = static_cast<size_t>(kt) * 2 * kWave;
        load_to_lds(bsrc + f, &S.b[wn][wm][0][0]);
        load_to_lds(bsrc + f + kWave, &S.b[wn][wm][1][0]);
    };

    f32x16 acc[NRB > 0 ? NRB : 1][2];
#pragma unroll
    for (int i = 0; i < NRB; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x16{0};

    // where this lane's A operand (row m = lane%32, k chunk 2*ks + lane/32) sits in
    // a staged row block: see the staging layout in the kernel below
    const int a_half = (lane % 32) / 16, a_r = lane % 16;
    const int a_pos[2] = {a_r * 4 + ((lane / 32) ^ ((a_r / 4) & 3)),
                          a_r * 4 + ((2 + lane / 32) ^ ((a_r / 4) & 3))};
    constexpr int NA = NRB > 0 ? NRB : 1;
    constexpr int kReads = NRB > 0 ? NRB + 2 : 0;   // LDS reads per half step
    auto read_frags = [&](int kt, int ks, bf16x8 (&a)[NA], bf16x8 (&b)[2]) {
        if (NRB == 0) return;
        const TiledStage& S = st[kt % kTiledStages];
        b[0] = S.b[wn][0][ks][lane];
        b[1] = S.b[wn][1][ks][lane];
#pragma unroll
        for (int i = 0; i < NRB; ++i) a[i] = S.a[2 * i + wm][a_half][a_pos[ks]];
    };
    auto multiply = [&](const bf16x8 (&a)[NA], const bf16x8 (&b)[2]) {
#pragma unroll
        for (int i = 0; i < NRB; ++i) {
            acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[0], acc[i][0], 0, 0, 0);
            acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[1], acc[i][1], 0, 0, 0);
        }
    };

    // Software pipeline: while the matrix cores work on one half (16 k) of a
    // step, the LDS reads of the next half are in flight.  A step's loads are
    // awaited (vmcnt) and published (barrier) half a step before it is needed;
    // the same barrier tells that every wave is done with the stage refilled next.
    constexpr int kAhead = kTiledStages - 1;            // steps in flight
#pragma unroll
    for (int q = 0; q < kAhead; ++q)
        if (q < KT) issue(q, q);
    // wait for step 0: everything issued after it may stay in flight
    if (KT >= kAhead)
        wait_vmcnt_le<(kAhead - 1) * kTiledLoadsPerStep>();
    else
        wait_vmcnt_le<0>();
    wg_barrier_nofence();
    bf16x8 a0[NA], b0[2], a1[NA], b1[2];
    // One half step = multiply the fragments read during the previous half
    // while reading the next half's: the scheduler is told to alternate one MFMA
    // with one LDS read, so the reads are issued under the first MFMAs and have
    // landed when the block of 2*NRB MFMAs (32 cycles each) is through.
    auto half_step = [&](int rd_kt, int rd_ks, bf16x8 (&ra)[NA], bf16x8 (&rb)[2],
                         const bf16x8 (&ma)[NA], const bf16x8 (&mb)[2]) {
        read_frags(rd_kt, rd_ks, ra, rb);
        multiply(ma, mb);
#pragma unroll
        for (int i = 0; i < kReads; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * NA, 0);  // the remaining MFMAs
        __builtin_amdgcn_sched_barrier(0);
    };

    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): no scalar load pending in the loop
    read_frags(0, 0, a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    int kt = 0;
    for (; kt + kAhead < KT; ++kt) {     // steady state: no branches inside
        half_step(kt, 1, a1, b1, a0, b0);
        // step kt+1 has landed once only the later steps' loads are outstanding
        wait_vmcnt_le<(kAhead - 2) * kTiledLoadsPerStep>();
        wg_barrier_nofence();
        issue(kt + kAhead, (kt + kAhead) % kTiledStages);
        __builtin_amdgcn_sched_barrier(0);
        half_step(kt + 1, 0, a0, b0, a1, b1);
    }
    for (; kt + 1 < KT; ++kt) {          // drain: nothing left to issue
        half_step(kt, 1, a1, b1, a0, b0);
        wait_vmcnt_le<0>();
        wg_barrier_nofence();
        __builtin_amdgcn_sched_barrier(0);
        half_step(kt + 1, 0, a0, b0, a1, b1);
    }
    half_step(kt, 1, a1, b1, a0, b0);    // last step
    multiply(a1, b1);

    // epilogue: lane l, register r -> row 8*(r/4) + 4*(l/32) + r%4, column l%32
    const int col = lane % 32;
#pragma unroll
    for (int i = 0; i < NRB; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = (2 * i + wm) * 32 + acc_row(r, lane);
            if (m >= rows) continue;
            if (SWIGLU) {
                const float av = acc[i][0][r], bv = acc[i][1][r];
                const size_t off = static_cast<size_t>(row0 + m) * ldc + nt * 128 + wn * 32 + col;
                static_cast<bf16_t*>(C)[off] = f32_to_bf16((av / (1.f + __expf(-av))) * bv);
            } else {
                const size_t off = static_cast<size_t>(row0 + m) * ldc + nt * 256 + wn * 64 + col;
                static_cast<float*>(C)[off] = acc[i][0][r];
                static_cast<float*>(C)[off + 32] = acc[i][1][r];
            }
        }
    }
}

template <bool SWIGLU>
__global__ __launch_bounds__(kTiledWaves* kWave, 1) void ffn_bf16_tiled_kernel(StreamGroup g0,
                                                                              StreamGroup g1) {
    __shared__ TiledStage st[kTiledStages];

    // Work order.  The hardware deals workgroups to the 8 XCDs round-robin by
    // blockIdx, and each XCD has its own L2.  Row tiles are taken in groups of 8:
    // inside a group, workgroup index 8*nt + x is (row tile 8g + x, column tile
    // nt), so XCD x runs every column tile of "its" row tile back to back and the
    // gathered A rows are fetched into one L2 only (measured: 21% less fabric
    // traffic and 3-6% less time than tile-major order).  The routed experts'
    // tiles come first, then the shared expert's.
    constexpr int kColsPerTile = SWIGLU ? 128 : 256;   // SwiGLU columns, or plain columns
    auto tiles_of = [](const StreamGroup& q) -> int {
        if (q.A == nullptr) return 0;
        return q.tile_info ? q.tile_info[0] : (q.M_dense + kTiledRows - 1) / kTiledRows;
    };
    const int tiles0 = tiles_of(g0), tiles1 = tiles_of(g1);
    const int nt0 = g0.A ? g0.N / kColsPerTile : 1, nt1 = g1.A ? g1.N / kColsPerTile : 1;
    const int64_t wg0 = static_cast<int64_t>((tiles0 + kXcds - 1) / kXcds * kXcds) * nt0;
    const bool first = static_cast<int64_t>(blockIdx.x) < wg0;
    const StreamGroup& g = first ? g0 : g1;
    const int64_t bid = first ? blockIdx.x : blockIdx.x - wg0;
    const int n_tiles = first ? nt0 : nt1;
    const int tile = static_cast<int>(bid / (kXcds * n_tiles)) * kXcds + static_cast<int>(bid % kXcds);
    const int nt = static_cast<int>(bid % (kXcds * n_tiles)) / kXcds;
    if (tile >= (first ? tiles0 : tiles1)) return;   // the grid is sized for the host's bound

    const bf16_t* __restrict__ A = static_cast<const bf16_t*>(g.A);
    const bf16_t* __restrict__ Bp = static_cast<const bf16_t*>(g.Bp);
    const int32_t* __restrict__ row_map = g.row_map;
    const int32_t* __restrict__ tile_info = g.tile_info;
    const int lda = g.lda, Kd = g.Kd, ldc = g.ldc, M_dense = g.M_dense;
    int e, row0, rows;
    if (tile_info != nullptr) {
        const int32_t* ent = tile_info + 4 + 4 * static_cast<size_t>(tile);
        e = ent[0];
        row0 = ent[1];
        rows = ent[2];
    } else {
        e = 0;
        row0 = tile * kTiledRows;
        rows = min(kTiledRows, M_dense - row0);
    }
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int wm = wave / 4, wn = wave % 4;
    const int n_rb = (rows + 31) / 32;              // row blocks that hold real rows
    const int my_rb = (n_rb - wm + 1) / 2;          // of those, this wave's (wm, wm+2, ...)
    const int KT = Kd / kTiledK;

    // A: this wave stages row block `wave` (32 rows x 32 k per step) with two
    // loads of 16 rows x 64 bytes: lanes 4r..4r+3 fetch the four 16-byte k chunks
    // of row r, so each lane quad reads 64 contiguous bytes.  Lane i's data lands
    // at position i of the 1 KB piece; it fetches chunk (i%4) ^ ((r/4)%4), an XOR
    // swizzle that spreads the MFMA operand reads (row m, chunk c at position
    // 4 (m%16) + (c ^ ((m%16)/4 % 4))) over all LDS banks.  Rows past the tile's
    // end re-read its last row (in bounds; their products are never stored).
    const bf16x8* arow[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = lane / 4;
        const int my_row = row0 + min(wave * 32 + j * 16 + r, rows - 1);
        const long src = row_map ? row_map[my_row] : my_row;
        arow[j] = reinterpret_cast<const bf16x8*>(A + static_cast<size_t>(src) * lda) +
                  ((lane % 4) ^ ((r / 4) & 3));
    }
    // B: this wave stages stream wm of column block wn: W1 (wm = 0) or W3 (wm = 1)
    // of SwiGLU column block 4 nt + wn, or W2's column block 8 nt + 2 wn + wm;
    // a stream is Kd/16 fragments of 64 x 16 B, contiguous
    const size_t stream_elems = static_cast<size_t>(Kd) * 32;
    const size_t sidx = SWIGLU ? static_cast<size_t>(4 * nt + wn) * 2 + wm
                               : static_cast<size_t>(8 * nt + 2 * wn + wm);
    const bf16x8* bsrc = reinterpret_cast<const bf16x8*>(
                             Bp + static_cast<size_t>(e) * g.group_stride + sidx * stream_elems) + lane;

    switch (my_rb) {   // uniform over the wave; every variant runs the same KT barriers
        case 4: tiled_body<SWIGLU, 4>(st, arow[0], arow[1], bsrc, KT, wm, wn, lane, row0, rows, nt, g.C, ldc); break;
        case 3: tiled_body<SWIGLU, 3>(st, arow[0], arow[1], bsrc, KT, wm, wn, lane, row0, rows, nt, g.C, ldc); break;
        case 2: tiled_body<SWIGLU, 2>(st, arow[0], arow[1], bsrc, KT, wm, wn, lane, row0, rows, nt, g.C, ldc); break;
        case 1: tiled_body<SWIGLU, 1>(st, arow[0], arow[1], bsrc, KT, wm, wn, lane, row0, rows, nt, g.C, ldc); break;
        default: tiled_body<SWIGLU, 0>(st, arow[0], arow[1], bsrc, KT, wm, wn, lane, row0, rows, nt, g.C, ldc); break;
    }
}

hipError_t launch_ffn_bf16_tiled(bool swiglu, StreamGroup routed, StreamGroup shared,
                                 hipStream_t stream) {
    const int cols = swiglu ? 128 : 256;
    auto count = [cols](StreamGroup& g) {
        int64_t tiles =
            g.A == nullptr ? 0 : (g.tile_info ? g.max_tiles : (g.M_dense + kTiledRows - 1) / kTiledRows);
        tiles = (tiles + kXcds - 1) / kXcds * kXcds;   // whole groups of 8 row tiles
        g.n_wg = tiles * (g.N / cols);
    };
    count(routed);   // an upper bound: the real tile count is known on the device only
    count(shared);
    const int64_t total = routed.n_wg + shared.n_wg;
    if (total <= 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>(total)), block(kTiledWaves * kWave);
    if (swiglu)
        hipLaunchKernelGGL(ffn_bf16_tiled_kernel<true>, grid, block, 0, stream, routed, shared);
    else
        hipLaunchKernelGGL(ffn_bf16_tiled_kernel<false>, grid, block, 0, stream, routed, shared);
    return hipGetLastError();
}

hipError_t launch_ffn_bf16_stream(bool swiglu, StreamGroup routed, StreamGroup shared,
                                  hipStream_t stream) {
    auto count = [](StreamGroup& g) {
        const int64_t tiles = g.A == nullptr ? 0 : (g.tile_info ? g.max_tiles : (g.M_dense + 31) / 32);
        g.n_wg = tiles * (g.N / 32);
    };
    count(routed);
    count(shared);
    const int64_t total = routed.n_wg + shared.n_wg;
    if (total <= 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>(total)), block(kStreamWaves * kWave);
    if (swiglu)
        hipLaunchKernelGGL(ffn_bf16_stream_kernel<true>, grid, block, 0, stream, routed, shared);
    else
        hipLaunchKernelGGL(ffn_bf16_stream_kernel<false>, grid, block, 0, stream, routed, shared);
    return hipGetLastError();
}

}  // namespace allocmoe
