// Measurement utilities: the two ceilings a roofline of the layer's kernels is
// judged against, re-measured on the device at hand.  Not on the layer's path.
//
//  * matrix-core issue loop: v_mfma_f32_32x32x16_bf16 back to back on eight
//    independent accumulators per wave, one or two waves per SIMD on every
//    compute unit, operands taken from a caller-filled buffer (zeros or random
//    values: the sustained clock, and with it the rate, depends on the data);
//    the shader clock is read as the ratio of the core-clock counter to the
//    constant 100 MHz counter around the loop.
//  * streaming read: every lane loads 16 bytes at a time, eight loads in flight,
//    a workgroup per contiguous 256 KB, with or without the non-temporal hint.
#include "../../include/allocmoe.h"

#include <hip/hip_runtime.h>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kProbeGrid = 256;        // one workgroup per compute unit
constexpr int kFragsPerLane = 6;       // 4 + 2 operand fragments of 16 bytes

template <int THREADS>
__global__ __launch_bounds__(THREADS) void mfma_probe_kernel(const bf16x8* __restrict__ operands,
                                                            int iters, float* __restrict__ sink,
                                                            long long* __restrict__ clocks) {
    const size_t me = static_cast<size_t>(blockIdx.x) * THREADS + threadIdx.x;
    bf16x8 a[4], b[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) a[j] = operands[me * kFragsPerLane + j];
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = operands[me * kFragsPerLane + 4 + j];
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x16{0};
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j % 4], b[j / 4], acc[j], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    sink[me] = s;
    if (threadIdx.x == 0) {
        clocks[2 * blockIdx.x] = c1 - c0;
        clocks[2 * blockIdx.x + 1] = w1 - w0;
    }
}

constexpr int kReadChunk = 256 * 1024;   // bytes per workgroup

template <bool NT>
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const u32x4* __restrict__ p,
                                                             uint32_t* __restrict__ sink) {
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const u32x4* base = p + static_cast<size_t>(blockIdx.x) * (kReadChunk / 16);
    u32x4 acc = {0, 0, 0, 0};
    for (int it = 0; it < 8; ++it) {   // 8 batches x 8 loads x 4 waves x 1 KB
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const u32x4* q = base + static_cast<size_t>(it * 8 + u) * 256 + wave * 64 + lane;
            v[u] = NT ? __builtin_nontemporal_load(q) : *q;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    // (practically never true: keeps the loads alive without a store per lane)
    if (acc[0] == 0x12345678u && acc[1] == 0x9abcdef0u) sink[0] = acc[2] ^ acc[3];
}

inline allocmoe_status hip_status(hipError_t e) { return e == hipSuccess ? ALLOCMOE_OK : ALLOCMOE_EHIP; }
#define PROBE_TRY(expr)                                   \
    do {                                                  \
        const allocmoe_status st_ = hip_status(expr);     \
        if (st_ != ALLOCMOE_OK) return st_;               \
    } while (0)

}  // namespace

extern "C" {

size_t allocmoe_probe_mfma_operand_bytes(void) {
    return static_cast<size_t>(kProbeGrid) * 512 * kFragsPerLane * 16;
}

size_t allocmoe_probe_sink_bytes(void) {
    return static_cast<size_t>(kProbeGrid) * 512 * 4 + static_cast<size_t>(kProbeGrid) * 16;
}

allocmoe_status allocmoe_probe_mfma(const void* operands, size_t operand_bytes, int waves_per_simd,
                                    int iters, void* sink, size_t sink_bytes, float* tflops,
                                    float* shader_mhz, allocmoe_stream stream_) {
    if (!operands || !sink || !tflops || !shader_mhz || iters < 1) return ALLOCMOE_EINVAL;
    if (waves_per_simd != 1 && waves_per_simd != 2) return ALLOCMOE_EINVAL;
    if (operand_bytes < allocmoe_probe_mfma_operand_bytes() || sink_bytes < allocmoe_probe_sink_bytes() ||
        reinterpret_cast<uintptr_t>(operands) % 16 || reinterpret_cast<uintptr_t>(sink) % 16)
        return ALLOCMOE_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    float* out = static_cast<float*>(sink);
    long long* clocks = reinterpret_cast<long long*>(out + static_cast<size_t>(kProbeGrid) * 512);
    const bf16x8* ops = static_cast<const bf16x8*>(operands);
    hipEvent_t e0, e1;
    PROBE_TRY(hipEventCreate(&e0));
    PROBE_TRY(hipEventCreate(&e1));
    auto launch = [&](int n) {
        if (waves_per_simd == 1)
            hipLaunchKernelGGL(mfma_probe_kernel<256>, dim3(kProbeGrid), dim3(256), 0, stream, ops, n, out, clocks);
        else
            hipLaunchKernelGGL(mfma_probe_kernel<512>, dim3(kProbeGrid), dim3(512), 0, stream, ops, n, out, clocks);
        return hipGetLastError();
    };
    PROBE_TRY(launch(64));   // warm-up
    PROBE_TRY(hipEventRecord(e0, stream));
    PROBE_TRY(launch(iters));
    PROBE_TRY(hipEventRecord(e1, stream));
    PROBE_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
    long long h[2 * kProbeGrid];
    PROBE_TRY(hipMemcpyAsync(h, clocks, sizeof(h), hipMemcpyDeviceToHost, stream));
    PROBE_TRY(hipStreamSynchronize(stream));
    double core = 0, wall = 0;
    for (int i = 0; i < kProbeGrid; ++i) {
        core += static_cast<double>(h[2 * i]);
        wall += static_cast<double>(h[2 * i + 1]);
    }
    const double flops = static_cast<double>(kProbeGrid) * 4 * waves_per_simd * iters * 8.0 * 32768.0;
    *tflops = static_cast<float>(flops / (ms * 1e-3) / 1e12);
    *shader_mhz = wall > 0 ? static_cast<float>(core / wall * 100.0) : 0.f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ALLOCMOE_OK;
}

allocmoe_status allocmoe_probe_hbm_read(const void* buf, size_t bytes, int nontemporal, int repeats,
                                        void* sink, size_t sink_bytes, float* gbytes_per_s,
                                        allocmoe_stream stream_) {
    if (!buf || !sink || !gbytes_per_s || repeats < 1) return ALLOCMOE_EINVAL;
    if (bytes < kReadChunk || sink_bytes < 16 || reinterpret_cast<uintptr_t>(buf) % 16)
        return ALLOCMOE_EWORKSPACE;
    const size_t groups = bytes / kReadChunk;
    if (groups > 0x7FFFFFFFu) return ALLOCMOE_ESHAPE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const u32x4* p = static_cast<const u32x4*>(buf);
    uint32_t* out = static_cast<uint32_t*>(sink);
    hipEvent_t e0, e1;
    PROBE_TRY(hipEventCreate(&e0));
    PROBE_TRY(hipEventCreate(&e1));
    auto launch = [&]() {
        if (nontemporal)
            hipLaunchKernelGGL(hbm_read_probe_kernel<true>, dim3(static_cast<unsigned>(groups)), dim3(256), 0, stream, p, out);
        else
            hipLaunchKernelGGL(hbm_read_probe_kernel<false>, dim3(static_cast<unsigned>(groups)), dim3(256), 0, stream, p, out);
        return hipGetLastError();
    };
    PROBE_TRY(launch());   // warm-up
    PROBE_TRY(hipEventRecord(e0, stream));
    for (int i = 0; i < repeats; ++i) PROBE_TRY(launch());
    PROBE_TRY(hipEventRecord(e1, stream));
    PROBE_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
    *gbytes_per_s = static_cast<float>(static_cast<double>(groups) * kReadChunk * repeats / (ms * 1e-3) / 1e9);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ALLOCMOE_OK;
}

}  // extern "C"
