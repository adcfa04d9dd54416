// Score-weighted combine (Section 3.1, Eq. (2)): y_t = sum_i w_{t,i} E_i(x_t)
// over the kept pairs of token t, the weight being the retained routing score
// (no renormalisation), plus the always-on shared expert's output times its
// gate.  A gather: one workgroup per token walks the token's kept ranks in
// order j = 0, 1, ... and adds s[t,j] * O[inv_row[t,j], :] in fp32, then the
// shared term, then rounds once to the output type.  A kept rank without a row
// (inv_row < 0: only possible when a caller hands the dispatch keep counts that sum
// to more than the budget) contributes nothing.
#include "common.hpp"
#include "kernels.hpp"

namespace allocmoe {

// 4 consecutive elements of a row as floats
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const bf16_t* p) {
    const uint2 v = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u),
                       __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xFFFF0000u));
}
__device__ __forceinline__ void store4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void store4(bf16_t* p, float4 v) {
    uint2 w;
    w.x = static_cast<uint32_t>(f32_to_bf16(v.x)) | (static_cast<uint32_t>(f32_to_bf16(v.y)) << 16);
    w.y = static_cast<uint32_t>(f32_to_bf16(v.z)) | (static_cast<uint32_t>(f32_to_bf16(v.w)) << 16);
    *reinterpret_cast<uint2*>(p) = w;
}

// TE: element type of the experts' outputs O, Os and of Y (the layer's dtype); the
// weighted sum itself is formed in fp32, in candidate order, shared expert last
template <typename TE>
__global__ __launch_bounds__(256) void combine_kernel(
    const TE* __restrict__ O, const TE* __restrict__ Os, const int32_t* __restrict__ inv_row,
    const float* __restrict__ topk_s, const int32_t* __restrict__ keep_count,
    const float* __restrict__ sgate, int T, int d, int K, TE* __restrict__ Y) {
    const int t = blockIdx.x;
    if (t >= T) return;
    const int kt = min(K, keep_count[t]);
    const int32_t* rows = inv_row + static_cast<size_t>(t) * K;
    const float* wts = topk_s + static_cast<size_t>(t) * K;
    const float g = Os ? (sgate ? sgate[t] : 1.f) : 0.f;
    if (sizeof(TE) == 2 && (d & 7) == 0) {
        // bf16: 8 elements (16 bytes) per lane and row
        for (int c = threadIdx.x * 8; c < d; c += blockDim.x * 8) {
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            auto add = [&](const TE* row, float wgt) {
                const uint4 v = *reinterpret_cast<const uint4*>(row + c);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[2 * i] += wgt * __uint_as_float(w[i] << 16);
                    acc[2 * i + 1] += wgt * __uint_as_float(w[i] & 0xFFFF0000u);
                }
            };
            for (int j = 0; j < kt; ++j)
                if (rows[j] >= 0) add(O + static_cast<size_t>(rows[j]) * d, wts[j]);
            if (Os) add(Os + static_cast<size_t>(t) * d, g);
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = static_cast<uint32_t>(f32_to_bf16(acc[2 * i])) |
                       (static_cast<uint32_t>(f32_to_bf16(acc[2 * i + 1])) << 16);
            *reinterpret_cast<uint4*>(Y + static_cast<size_t>(t) * d + c) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    } else if ((d & 3) == 0) {
        for (int c = threadIdx.x * 4; c < d; c += blockDim.x * 4) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int j = 0; j < kt; ++j) {
                if (rows[j] < 0) continue;
                const float4 o = load4(O + static_cast<size_t>(rows[j]) * d + c);
                acc.x += wts[j] * o.x;
                acc.y += wts[j] * o.y;
                acc.z += wts[j] * o.z;
                acc.w += wts[j] * o.w;
            }
            if (Os) {
                const float4 o = load4(Os + static_cast<size_t>(t) * d + c);
                acc.x += g * o.x;
                acc.y += g * o.y;
                acc.z += g * o.z;
                acc.w += g * o.w;
            }
            store4(Y + static_cast<size_t>(t) * d + c, acc);
        }
    } else {
        for (int c = threadIdx.x; c < d; c += blockDim.x) {
            float acc = 0.f;
            for (int j = 0; j < kt; ++j)
                if (rows[j] >= 0) acc += wts[j] * load_f32(O, static_cast<size_t>(rows[j]) * d + c);
            if (Os) acc += g * load_f32(Os, static_cast<size_t>(t) * d + c);
            store_elem(Y, static_cast<size_t>(t) * d + c, acc);
        }
    }
}

hipError_t launch_combine(int dtype, const void* O, const void* Os, const int32_t* inv_row,
                          const float* topk_s, const int32_t* keep_count, const float* sgate,
                          int T, int d, int K, void* Y, hipStream_t stream) {
    const dim3 grid(T), block(256);
    if (dtype == 0)
        hipLaunchKernelGGL(combine_kernel<float>, grid, block, 0, stream,
                           static_cast<const float*>(O), static_cast<const float*>(Os), inv_row,
                           topk_s, keep_count, sgate, T, d, K, static_cast<float*>(Y));
    else
        hipLaunchKernelGGL(combine_kernel<bf16_t>, grid, block, 0, stream,
                           static_cast<const bf16_t*>(O), static_cast<const bf16_t*>(Os), inv_row,
                           topk_s, keep_count, sgate, T, d, K, static_cast<bf16_t*>(Y));
    return hipGetLastError();
}

}  // namespace allocmoe
