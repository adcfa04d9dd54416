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
// A workgroup (4 waves) owns a tile of <= 128 rows of one expert times 128
// SwiGLU columns (128 of W1 and the same 128 of W3; for the second GEMM: 256
// columns of W2).  Wave w owns all the tile's rows times column block w (32
// W1-columns + 32 W3-columns, or 2 x 32 W2-columns): 4 x 2 MFMA accumulators of
// 32x32.  The contraction runs in steps of 32 through a 3-stage LDS ring that is
// filled by direct-to-LDS loads (16 B per lane, 1 KB per wave-load, no VGPR
// staging): A fragments are gathered row by row straight into MFMA operand
// order, the re-tiled weights are already in that order, so every fragment is
// read back with one conflict-free ds_read_b128.  Loads of step kt+2 are in
// flight while step kt is multiplied; one barrier per step.
constexpr int kTiledRows = 128;
constexpr int kTiledK = 32;
constexpr int kTiledStages = 3;
constexpr int kTiledLoadsPerStep = 6;   // per wave: 2 A fragments + 4 B fragments

struct alignas(16) TiledStage {
    bf16x8 a[4][2][kWave];      // [row block][k16 half][lane]
    bf16x8 b[4][2][2][kWave];   // [wave][stream][k16 half][lane]
};

__device__ __forceinline__ void load_to_lds(const bf16x8* gptr, bf16x8* lds_frag) {
    // lane l's 16 bytes land at lds_frag + l (hardware adds lane * 16 to the base)
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

// Main loop and epilogue for a tile with NRB row blocks of 32 holding real rows.
template <bool SWIGLU, int NRB>
__device__ __forceinline__ void tiled_body(TiledStage* st, const bf16x8* ap, const bf16x8* bs0,
                                           const bf16x8* bs1, int KT, int wave, int lane,
                                           int row0, int rows, int nt, void* C, int ldc) {
    auto issue = [&](int kt, int stage) {
        TiledStage& S = st[stage];
        load_to_lds(ap + kt * 4, &S.a[wave][0][0]);
        load_to_lds(ap + kt * 4 + 2, &S.a[wave][1][0]);
        const size_t f = static_cast<size_t>(kt) * 2 * kWave;
        load_to_lds(bs0 + f, &S.b[wave][0][0][0]);
        load_to_lds(bs0 + f + kWave, &S.b[wave][0][1][0]);
        load_to_lds(bs1 + f, &S.b[wave][1][0][0]);
        load_to_lds(bs1 + f + kWave, &S.b[wave][1][1][0]);
    };

    f32x16 acc[NRB][2];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[rb][j] = f32x16{0};

    issue(0, 0);
    if (KT > 1) issue(1, 1);
    for (int kt = 0; kt < KT; ++kt) {
        // this wave's loads of step kt have landed once at most the loads of
        // step kt+1 are outstanding; the barrier then publishes every wave's part
        // and tells that everyone is done reading the stage refilled next
        if (kt + 1 < KT)
            __builtin_amdgcn_s_waitcnt(0xF70 | kTiledLoadsPerStep);   // vmcnt <= 6
        else
            __builtin_amdgcn_s_waitcnt(0xF70);                        // vmcnt == 0
        wg_barrier_nofence();
        if (kt + 2 < KT) issue(kt + 2, (kt + 2) % kTiledStages);
        const TiledStage& S = st[kt % kTiledStages];
        bf16x8 a[2][NRB], b[2][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            b[ks][0] = S.b[wave][0][ks][lane];
            b[ks][1] = S.b[wave][1][ks][lane];
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) a[ks][rb] = S.a[rb][ks][lane];
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) {
                acc[rb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][rb], b[ks][0], acc[rb][0], 0, 0, 0);
                acc[rb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][rb], b[ks][1], acc[rb][1], 0, 0, 0);
            }
    }

    // epilogue: lane l, register r -> row 8*(r/4) + 4*(l/32) + r%4, column l%32
    const int col = lane % 32;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = rb * 32 + acc_row(r, lane);
            if (m >= rows) continue;
            if (SWIGLU) {
                const float av = acc[rb][0][r], bv = acc[rb][1][r];
                const size_t off = static_cast<size_t>(row0 + m) * ldc + nt * 128 + wave * 32 + col;
                static_cast<bf16_t*>(C)[off] = f32_to_bf16((av / (1.f + __expf(-av))) * bv);
            } else {
                const size_t off = static_cast<size_t>(row0 + m) * ldc + nt * 256 + wave * 64 + col;
                static_cast<float*>(C)[off] = acc[rb][0][r];
                static_cast<float*>(C)[off + 32] = acc[rb][1][r];
            }
        }
    }
}

template <bool SWIGLU>
__global__ __launch_bounds__(256, 2) void ffn_bf16_tiled_kernel(StreamGroup g0, StreamGroup g1) {
    __shared__ TiledStage st[kTiledStages];

    const bool first = static_cast<int64_t>(blockIdx.x) < g0.n_wg;
    const StreamGroup& g = first ? g0 : g1;
    const int bid = first ? blockIdx.x : blockIdx.x - static_cast<unsigned>(g0.n_wg);
    const bf16_t* __restrict__ A = static_cast<const bf16_t*>(g.A);
    const bf16_t* __restrict__ Bp = static_cast<const bf16_t*>(g.Bp);
    const int32_t* __restrict__ row_map = g.row_map;
    const int32_t* __restrict__ tile_info = g.tile_info;
    const int lda = g.lda, Kd = g.Kd, N = g.N, ldc = g.ldc, M_dense = g.M_dense;

    // column tiles: 128 SwiGLU columns (of W1 and of W3) or 256 plain columns
    constexpr int kColsPerTile = SWIGLU ? 128 : 256;
    const int n_tiles = N / kColsPerTile;
    const int tile = bid / n_tiles, nt = bid % n_tiles;
    int e, row0, rows;
    if (tile_info != nullptr) {
        if (tile >= tile_info[0]) return;
        const int32_t* ent = tile_info + 4 + 4 * static_cast<size_t>(tile);
        e = ent[0];
        row0 = ent[1];
        rows = ent[2];
    } else {
        e = 0;
        row0 = tile * kTiledRows;
        if (row0 >= M_dense) return;
        rows = min(kTiledRows, M_dense - row0);
    }
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int n_rb = (rows + 31) / 32;          // row blocks that hold real rows
    const int KT = Kd / kTiledK;

    // A: this wave stages row block `wave`; lane (m = l%32, kg = l/32) fetches 8
    // consecutive k of its row.  Rows past the tile's end re-read its last row
    // (in bounds; their products are never stored).
    const int my_row = row0 + min(wave * 32 + lane % 32, rows - 1);
    const long src = row_map ? row_map[my_row] : my_row;
    const bf16x8* ap =
        reinterpret_cast<const bf16x8*>(A + static_cast<size_t>(src) * lda) + lane / 32;
    // B: two fragment streams per wave (W1 and W3 of column block 4 nt + wave, or
    // W2's column blocks 8 nt + 2 wave and + 1), each Kd/16 fragments of 64 x 16 B
    const size_t stream_elems = static_cast<size_t>(Kd) * 32;
    const size_t cb = SWIGLU ? static_cast<size_t>(4 * nt + wave) * 2
                             : static_cast<size_t>(8 * nt + 2 * wave);
    const bf16x8* bs0 = reinterpret_cast<const bf16x8*>(
                            Bp + static_cast<size_t>(e) * g.group_stride + cb * stream_elems) + lane;
    const bf16x8* bs1 = bs0 + stream_elems / 8;

    switch (n_rb) {   // uniform over the workgroup
        case 4: tiled_body<SWIGLU, 4>(st, ap, bs0, bs1, KT, wave, lane, row0, rows, nt, g.C, ldc); break;
        case 3: tiled_body<SWIGLU, 3>(st, ap, bs0, bs1, KT, wave, lane, row0, rows, nt, g.C, ldc); break;
        case 2: tiled_body<SWIGLU, 2>(st, ap, bs0, bs1, KT, wave, lane, row0, rows, nt, g.C, ldc); break;
        default: tiled_body<SWIGLU, 1>(st, ap, bs0, bs1, KT, wave, lane, row0, rows, nt, g.C, ldc); break;
    }
}

hipError_t launch_ffn_bf16_tiled(bool swiglu, StreamGroup routed, StreamGroup shared,
                                 hipStream_t stream) {
    const int cols = swiglu ? 128 : 256;
    auto count = [cols](StreamGroup& g) {
        const int64_t tiles =
            g.A == nullptr ? 0 : (g.tile_info ? g.max_tiles : (g.M_dense + kTiledRows - 1) / kTiledRows);
        g.n_wg = tiles * (g.N / cols);
    };
    count(routed);
    count(shared);
    const int64_t total = routed.n_wg + shared.n_wg;
    if (total <= 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>(total)), block(256);
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
