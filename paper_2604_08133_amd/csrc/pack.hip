// One-time re-tiling of row-major bf16 weight matrices W[g][k][n] into the
// operand order of v_mfma_f32_32x32x16_bf16, so that the per-batch kernels load
// B fragments with one contiguous 16-byte load per lane.
//
// A fragment covers 16 k x 32 n: lane l holds the 8 values
//   W[16*kb + 8*(l/32) + i][32*nb + l%32],  i = 0..7,
// stored as 64 lanes x 16 bytes = 1 KB.  The fragments of one column block nb
// are contiguous along k (kb = 0 .. Kd/16-1).  Destination of fragment
// (g, nb, kb):  out + g*group_stride + nb*nblock_stride + base_off + kb*512.
#include "common.hpp"
#include "kernels.hpp"

namespace allocmoe {

__global__ __launch_bounds__(256) void pack_b_kernel(const bf16_t* __restrict__ W, int G, int Kd,
                                                     int N, bf16_t* __restrict__ out,
                                                     size_t group_stride, size_t nblock_stride,
                                                     size_t base_off) {
    const int KB = Kd / 16, NB = N / 32;
    const size_t total = static_cast<size_t>(G) * NB * KB * kWave;
    const size_t idx = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int l = idx % kWave;
    size_t f = idx / kWave;
    const int kb = f % KB;
    f /= KB;
    const int nb = f % NB;
    const int g = f / NB;
    const int n = nb * 32 + (l % 32), k0 = kb * 16 + 8 * (l / 32);
    const bf16_t* src = W + (static_cast<size_t>(g) * Kd + k0) * N + n;
    bf16_t* dst = out + static_cast<size_t>(g) * group_stride +
                  static_cast<size_t>(nb) * nblock_stride + base_off +
                  static_cast<size_t>(kb) * 512 + static_cast<size_t>(l) * 8;
    uint32_t packed[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t lo = src[static_cast<size_t>(2 * i) * N];
        const uint32_t hi = src[static_cast<size_t>(2 * i + 1) * N];
        packed[i] = lo | (hi << 16);
    }
    *reinterpret_cast<uint4*>(dst) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
}

hipError_t launch_pack_b(const void* W, int G, int Kd, int N, void* out,
                         size_t group_stride_elems, size_t nblock_stride_elems,
                         size_t base_off_elems, hipStream_t stream) {
    const size_t total = static_cast<size_t>(G) * (N / 32) * (Kd / 16) * kWave;
    if (total == 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>((total + 255) / 256)), block(256);
    hipLaunchKernelGGL(pack_b_kernel, grid, block, 0, stream, static_cast<const bf16_t*>(W), G, Kd,
                       N, static_cast<bf16_t*>(out), group_stride_elems, nblock_stride_elems,
                       base_off_elems);
    return hipGetLastError();
}

}  // namespace allocmoe
