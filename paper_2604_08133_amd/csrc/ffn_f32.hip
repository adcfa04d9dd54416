// fp32 expert networks (Section 3.1: one feed-forward execution per selected
// pair) for the small full-precision configuration: a plain LDS-tiled grouped
// GEMM on the vector ALUs, any d / I / N, fused SwiGLU epilogue
//   H = silu(A W1) * (A W3)      (swiglu)      or      O = A W2.
// Row tiles come from the tile map the plan kernel wrote (rows of one expert
// never share a tile with another expert).
#include "common.hpp"
#include "kernels.hpp"

namespace allocmoe {

constexpr int kF32BM = 32, kF32BN = 64, kF32BK = 16;

template <bool SWIGLU>
__global__ __launch_bounds__(256) void ffn_f32_kernel(
    const float* __restrict__ A, int lda, const int32_t* __restrict__ row_map,
    const float* __restrict__ B1, const float* __restrict__ B3, int Kd, int N,
    const int32_t* __restrict__ tile_info, int M_dense, float* __restrict__ C, int ldc) {
    __shared__ float As[kF32BK][kF32BM + 1];
    __shared__ float B1s[kF32BK][kF32BN];
    __shared__ float B3s[SWIGLU ? kF32BK : 1][kF32BN];

    // flat grid: block = tile * n_blocks + n_block
    const int n_blocks = (N + kF32BN - 1) / kF32BN;
    const int tile = blockIdx.x / n_blocks, n_block = blockIdx.x % n_blocks;
    int e, row0, rows;
    if (tile_info != nullptr) {
        if (tile >= tile_info[0]) return;
        const int32_t* ent = tile_info + kTileHdr + 4 * static_cast<size_t>(tile);
        e = ent[0];
        row0 = ent[1];
        rows = ent[2];
    } else {
        e = 0;
        row0 = tile * kF32BM;
        if (row0 >= M_dense) return;
        rows = min(kF32BM, M_dense - row0);
    }
    const int n0 = n_block * kF32BN;
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const float* b1 = B1 + static_cast<size_t>(e) * Kd * N;
    const float* b3 = SWIGLU ? B3 + static_cast<size_t>(e) * Kd * N : nullptr;

    // source rows of the two A elements this thread stages per K step
    const int am = tid / kF32BK, ak = tid % kF32BK;   // am in 0..15, second element am+16
    long arow[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int m = am + 16 * q;
        arow[q] = -1;
        if (m < rows) {
            const int r = row0 + m;
            arow[q] = row_map ? row_map[r] : r;
        }
    }

    float acc1[2][4] = {}, acc3[2][4] = {};
    for (int k0 = 0; k0 < Kd; k0 += kF32BK) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int k = k0 + ak;
            As[ak][am + 16 * q] =
                (arow[q] >= 0 && k < Kd) ? A[static_cast<size_t>(arow[q]) * lda + k] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = tid + 256 * q, k = idx / kF32BN, n = idx % kF32BN;
            const bool ok = (k0 + k < Kd) && (n0 + n < N);
            const size_t off = static_cast<size_t>(k0 + k) * N + n0 + n;
            B1s[k][n] = ok ? b1[off] : 0.f;
            if (SWIGLU) B3s[k][n] = ok ? b3[off] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kF32BK; ++k) {
            const float a0 = As[k][ty * 2], a1 = As[k][ty * 2 + 1];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float w1 = B1s[k][tx * 4 + j];
                acc1[0][j] += a0 * w1;
                acc1[1][j] += a1 * w1;
                if (SWIGLU) {
                    const float w3 = B3s[k][tx * 4 + j];
                    acc3[0][j] += a0 * w3;
                    acc3[1][j] += a1 * w3;
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = ty * 2 + i;
        if (m >= rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc1[i][j];
            if (SWIGLU) v = (v / (1.f + expf(-v))) * acc3[i][j];
            C[static_cast<size_t>(row0 + m) * ldc + n] = v;
        }
    }
}

hipError_t launch_ffn_f32(bool swiglu, const float* A, int lda, const int32_t* row_map,
                          const float* B1, const float* B3, int Kd, int N,
                          const int32_t* tile_info, int64_t max_tiles, int M_dense, float* C,
                          int ldc, hipStream_t stream) {
    const int64_t tiles = tile_info ? max_tiles : (M_dense + kF32BM - 1) / kF32BM;
    if (tiles <= 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>(tiles * ((N + kF32BN - 1) / kF32BN))), block(256);
    if (swiglu)
        hipLaunchKernelGGL(ffn_f32_kernel<true>, grid, block, 0, stream, A, lda, row_map, B1, B3,
                           Kd, N, tile_info, M_dense, C, ldc);
    else
        hipLaunchKernelGGL(ffn_f32_kernel<false>, grid, block, 0, stream, A, lda, row_map, B1, B3,
                           Kd, N, tile_info, M_dense, C, ldc);
    return hipGetLastError();
}

}  // namespace allocmoe
