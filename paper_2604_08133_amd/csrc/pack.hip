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

// ---- 8-bit expert weights (E4M3 codes, one fp32 scale per output column)

// E4M3 of the OCP 8-bit floating point format: sign, 4 exponent bits (bias 7), 3 mantissa
// bits, subnormals, no infinities, largest finite magnitude 448.  Nearest code, ties to
// the even mantissa, magnitudes above 448 saturate.
__device__ __forceinline__ uint32_t e4m3_encode(float y) {
    const uint32_t sign = (__float_as_uint(y) >> 24) & 0x80u;
    const float a = fminf(fabsf(y), 448.f);
    uint32_t code;
    if (a < 0.015625f) {                       // below the smallest normal 2^-6: steps of 2^-9
        code = static_cast<uint32_t>(__float2int_rn(a * 512.f));   // 8 = the smallest normal
    } else {
        const uint32_t u = __float_as_uint(a);
        uint32_t e = (u >> 23) - 120u;         // biased by 7: (exponent - 127) + 7
        uint32_t m = (u >> 20) & 7u;
        const uint32_t rest = u & 0xFFFFFu, half = 0x80000u;
        if (rest > half || (rest == half && (m & 1u))) ++m;
        code = (e << 3) + m;                   // a mantissa carry moves into the exponent
        code = min(code, 0x7Eu);
    }
    return sign | code;
}

__global__ __launch_bounds__(256) void column_scale_kernel(const bf16_t* __restrict__ W, int G,
                                                           int Kd, int N,
                                                           float* __restrict__ scale,
                                                           size_t scale_stride) {
    const size_t idx = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= static_cast<size_t>(G) * N) return;
    const int n = idx % N, g = idx / N;
    const bf16_t* src = W + static_cast<size_t>(g) * Kd * N + n;
    float amax = 0.f;
    for (int k = 0; k < Kd; ++k) amax = fmaxf(amax, fabsf(bf16_to_f32(src[static_cast<size_t>(k) * N])));
    scale[static_cast<size_t>(g) * scale_stride + n] = amax > 0.f ? __fdiv_rn(amax, 448.f) : 1.f;
}

__global__ __launch_bounds__(256) void pack_b_fp8_kernel(const bf16_t* __restrict__ W, int G, int Kd,
                                                         int N, uint8_t* __restrict__ out,
                                                         size_t group_stride, size_t nblock_stride,
                                                         size_t base_off,
                                                         const float* __restrict__ scale,
                                                         size_t scale_stride) {
    const int KB = Kd / 32, NB = N / 32;
    const size_t total = static_cast<size_t>(G) * NB * KB * kWave;
    const size_t idx = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int l = idx % kWave;
    size_t f = idx / kWave;
    const int kb = f % KB;
    f /= KB;
    const int nb = f % NB;
    const int g = f / NB;
    const int n = nb * 32 + (l % 32);
    const float sc = scale[static_cast<size_t>(g) * scale_stride + n];
    uint32_t words[4] = {0, 0, 0, 0};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int k0 = kb * 32 + 16 * h + 8 * (l / 32);
        const bf16_t* src = W + (static_cast<size_t>(g) * Kd + k0) * N + n;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float w = bf16_to_f32(src[static_cast<size_t>(i) * N]);
            words[2 * h + i / 4] |= e4m3_encode(__fdiv_rn(w, sc)) << (8 * (i % 4));
        }
    }
    uint8_t* dst = out + static_cast<size_t>(g) * group_stride +
                   static_cast<size_t>(nb) * nblock_stride + base_off +
                   static_cast<size_t>(kb) * 1024 + static_cast<size_t>(l) * 16;
    *reinterpret_cast<uint4*>(dst) = make_uint4(words[0], words[1], words[2], words[3]);
}

hipError_t launch_pack_b_fp8(const void* W, int G, int Kd, int N, void* out, size_t group_stride,
                             size_t nblock_stride, size_t base_off, float* scale_out,
                             size_t scale_stride, hipStream_t stream) {
    const size_t cols = static_cast<size_t>(G) * N;
    const size_t total = static_cast<size_t>(G) * (N / 32) * (Kd / 32) * kWave;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(column_scale_kernel, dim3(static_cast<unsigned>((cols + 255) / 256)),
                       dim3(256), 0, stream, static_cast<const bf16_t*>(W), G, Kd, N, scale_out,
                       scale_stride);
    hipLaunchKernelGGL(pack_b_fp8_kernel, dim3(static_cast<unsigned>((total + 255) / 256)),
                       dim3(256), 0, stream, static_cast<const bf16_t*>(W), G, Kd, N,
                       static_cast<uint8_t*>(out), group_stride, nblock_stride, base_off, scale_out,
                       scale_stride);
    return hipGetLastError();
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
