// bf16 expert networks on the matrix cores (Section 3.1: one feed-forward
// execution per selected pair), fp32 accumulation, from weights re-tiled once
// into MFMA fragment order (pack.hip):
//   H = silu(A W1) * (A W3)   (SWIGLU)    or    O = A W2,   both stored as bf16.
//
// Weight-streaming kernel.  For token counts where an expert sees only a few
// rows the layer is bound by reading each active expert's weights once from
// HBM.  A workgroup owns one (row tile of <= 32 rows, block of 32 output
// columns); its 4 waves split the contraction dimension, each streaming its
// share of the packed weight fragments straight from global memory into MFMA B
// operands (1 KB contiguous per wave-load, every byte read once), with many
// independent loads in flight.  The A operand (<= 32 activation rows, L2
// resident) is gathered per lane.  Partial accumulators meet in LDS in a fixed
// order, so results are bitwise reproducible.
#include <type_traits>

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

// 8 E4M3 codes (two dwords) -> 8 bf16 values, exactly (every E4M3 value is a bf16 value);
// byte i of the pair is element i
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(uint32_t lo, uint32_t hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
    const bf16x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
    const bf16x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
    const bf16x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 w = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1),
                     __builtin_bit_cast(uint32_t, p2), __builtin_bit_cast(uint32_t, p3)};
    return __builtin_bit_cast(bf16x8, w);
}

// FP8: the weights are E4M3 codes with one scale per output column (pack.hip): a lane's
// 16-byte load then holds its fragments of TWO k16 steps, the codes are widened to bf16
// in registers (exact) and the column scale multiplies the fp32 sum at the end.  The
// waves take blocks of 32 k round-robin; Kd must be a multiple of 128.
template <bool SWIGLU, bool FP8>
__global__ __launch_bounds__(kStreamWaves* kWave) void ffn_bf16_stream_kernel(StreamGroup g0,
                                                                             StreamGroup g1) {
    constexpr int NACC = SWIGLU ? 2 : 1;
    __shared__ float red[kStreamWaves][NACC][16][kWave];

    // The grid is the shared expert's workgroups followed by the routed group's: the
    // shared expert has few workgroups with a long stream each, which should start
    // at once and run beside the routed ones instead of forming the launch's tail.
    const bool dense = static_cast<int64_t>(blockIdx.x) < g1.n_wg;
    const StreamGroup& g = dense ? g1 : g0;
    const int bid = dense ? blockIdx.x : blockIdx.x - static_cast<unsigned>(g1.n_wg);
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
        const int32_t* ent = tile_info + kTileHdr + 4 * static_cast<size_t>(tile);
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
    constexpr int kStepK = FP8 ? 32 : 16;   // k per load
    const int KB = Kd / kStepK;             // loads per stream in total
    const int steps = KB / kStreamWaves;    // per wave (Kd is a multiple of 64; 128 with FP8)
    // The waves take the k16 steps round-robin (wave w: steps w, w+4, ...), so at
    // any time the workgroup reads one contiguous run of each weight stream.

    // packed B: for this expert and column block, KB fragments of 64 x bf16x8
    // (W1 stream, then for SWIGLU the W3 stream)
    // (a stream of one column block holds Kd * 32 elements: 2 bytes each, or 1 with FP8)
    const bf16x8* b1 = reinterpret_cast<const bf16x8*>(
                           reinterpret_cast<const char*>(Bp) +
                           (static_cast<size_t>(e) * group_stride +
                            static_cast<size_t>(nb) * (static_cast<size_t>(NACC) * Kd * 32)) *
                               (FP8 ? 1 : 2)) +
                       static_cast<size_t>(wave) * kWave + lane;
    const bf16x8* b3 = b1 + static_cast<size_t>(KB) * kWave;
    constexpr size_t kStepB = static_cast<size_t>(kStreamWaves) * kWave;   // fragments per round

    // A: lane (m = l%32, kg = l/32) reads 8 consecutive k of its row per step
    const int m = lane % 32, kg = lane / 32;
    const bool a_ok = m < rows;
    long src = 0;
    if (a_ok) {
        const int r = row0 + m;
        src = row_map ? row_map[r] : r;
    }
    const bf16x8* ap = reinterpret_cast<const bf16x8*>(A + static_cast<size_t>(src) * lda) +
                       wave * (kStepK / 8) + kg;
    constexpr int kStepA = kStreamWaves * (kStepK / 8);

    f32x16 acc1 = {0}, acc3 = {0};
    const bf16x8 zero = {0};
    // a batch of N steps: all loads first (they are in flight together), then the MFMAs
    auto batch = [&](int s, auto n_const) {
        constexpr int N = decltype(n_const)::value;
        bf16x8 av[N], av2[N], w1[N], w3[N];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            w1[u] = __builtin_nontemporal_load(b1 + static_cast<size_t>(s + u) * kStepB);
            if (SWIGLU) w3[u] = __builtin_nontemporal_load(b3 + static_cast<size_t>(s + u) * kStepB);
            av[u] = a_ok ? ap[(s + u) * kStepA] : zero;
            if (FP8) av2[u] = a_ok ? ap[(s + u) * kStepA + 2] : zero;
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            if (FP8) {
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                const u32x4 q1 = __builtin_bit_cast(u32x4, w1[u]);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[u], fp8x8_to_bf16x8(q1[0], q1[1]), acc1, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av2[u], fp8x8_to_bf16x8(q1[2], q1[3]), acc1, 0, 0, 0);
                if (SWIGLU) {
                    const u32x4 q3 = __builtin_bit_cast(u32x4, w3[u]);
                    acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[u], fp8x8_to_bf16x8(q3[0], q3[1]), acc3, 0, 0, 0);
                    acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av2[u], fp8x8_to_bf16x8(q3[2], q3[3]), acc3, 0, 0, 0);
                }
            } else {
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[u], w1[u], acc1, 0, 0, 0);
                if (SWIGLU) acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[u], w3[u], acc3, 0, 0, 0);
            }
        }
    };
    int s = 0;
    for (; s + kStreamUnroll <= steps; s += kStreamUnroll)
        batch(s, std::integral_constant<int, kStreamUnroll>{});
    static_assert(kStreamUnroll == 8, "the switch below lists the short last batches");
    switch (steps - s) {   // uniform
        case 7: batch(s, std::integral_constant<int, 7>{}); break;
        case 6: batch(s, std::integral_constant<int, 6>{}); break;
        case 5: batch(s, std::integral_constant<int, 5>{}); break;
        case 4: batch(s, std::integral_constant<int, 4>{}); break;
        case 3: batch(s, std::integral_constant<int, 3>{}); break;
        case 2: batch(s, std::integral_constant<int, 2>{}); break;
        case 1: batch(s, std::integral_constant<int, 1>{}); break;
        default: break;
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
        if (FP8) {   // the column scales
            const float* sc = g.scale + static_cast<size_t>(e) * NACC * N;
            v1 *= sc[n];
            if (SWIGLU) v3 *= sc[N + n];
        }
        if (mr < rows) {
            const size_t off = static_cast<size_t>(row0 + mr) * ldc + n;
            if (SWIGLU)
                static_cast<bf16_t*>(Cv)[off] = f32_to_bf16(v1 * v3 * __builtin_amdgcn_rcpf(1.f + __expf(-v1)));
            else
                static_cast<bf16_t*>(Cv)[off] = f32_to_bf16(v1);
        }
    }
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
    const bool fp8 = (routed.A ? routed.scale : shared.scale) != nullptr;
    if (routed.A && shared.A && (routed.scale != nullptr) != (shared.scale != nullptr))
        return hipErrorInvalidValue;   // one weight format per launch
    if (fp8 && ((routed.A && routed.Kd % 128) || (shared.A && shared.Kd % 128)))
        return hipErrorInvalidValue;
    if (swiglu && fp8)
        hipLaunchKernelGGL((ffn_bf16_stream_kernel<true, true>), grid, block, 0, stream, routed, shared);
    else if (swiglu)
        hipLaunchKernelGGL((ffn_bf16_stream_kernel<true, false>), grid, block, 0, stream, routed, shared);
    else if (fp8)
        hipLaunchKernelGGL((ffn_bf16_stream_kernel<false, true>), grid, block, 0, stream, routed, shared);
    else
        hipLaunchKernelGGL((ffn_bf16_stream_kernel<false, false>), grid, block, 0, stream, routed, shared);
    return hipGetLastError();
}

}  // namespace allocmoe
