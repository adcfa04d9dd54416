// Routing scores and per-token candidates (Section 3.1, Eq. (1); Section 3.3,
// Eq. (6)): logits = x W_gate (+bias), softmax over all E experts, then each
// token's K largest scores in descending order (ties: lower expert id).
//
// Layout: one lane per expert (E <= 64).  A workgroup of 4 waves owns kTok
// tokens; the waves split the hidden dimension, each lane accumulating the
// logit of its expert, and the partial sums meet in LDS in a fixed order.
#include "common.hpp"
#include "kernels.hpp"

namespace allocmoe {

constexpr int kRouteTok = 4;    // tokens per workgroup
constexpr int kRouteWaves = 4;  // waves per workgroup, splitting d

// Sorted Top-K of one token's scores, lane = expert: larger score first, equal
// scores lower expert first.  Every lane counts the lanes that precede it in
// that order (its rank), and the lanes with rank < K store their (expert, score)
// at position rank of the token's candidate row.
__device__ __forceinline__ void wave_topk_store(float score, bool valid, int K,
                                                int32_t* __restrict__ ids_row,
                                                float* __restrict__ s_row) {
    const int lane = lane_id();
    // valid lanes: key >= 1 (scores are >= 0, so ordered_key has its top bit set)
    const uint32_t key = valid ? ordered_key(score) : 0u;
    int rank = 0;
#pragma unroll
    for (int o = 0; o < kWave; ++o) {
        const uint32_t ko = __builtin_amdgcn_readlane(key, o);
        rank += (ko > key || (ko == key && o < lane)) ? 1 : 0;
    }
    if (valid && rank < K) {
        ids_row[rank] = lane;
        s_row[rank] = score;
    }
}

template <typename TIn>
__global__ __launch_bounds__(kRouteWaves* kWave) void route_kernel(
    const TIn* __restrict__ X, const TIn* __restrict__ Wg, const float* __restrict__ bias,
    const TIn* __restrict__ w_sg, int T, int d, int E, int K, float* __restrict__ scores,
    int32_t* __restrict__ topk_ids, float* __restrict__ topk_s, float* __restrict__ sgate) {
    __shared__ float part[kRouteWaves][kRouteTok][kWave];
    __shared__ float gpart[kRouteWaves][kRouteTok];

    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int t0 = blockIdx.x * kRouteTok;

    // this wave's slice of the hidden dimension, in chunks of 64
    const int chunks = (d + kWave - 1) / kWave;
    const int per_wave = (chunks + kRouteWaves - 1) / kRouteWaves;
    const int c_begin = wave * per_wave;
    const int c_end = min(chunks, c_begin + per_wave);

    float acc[kRouteTok];
    float gacc[kRouteTok];
#pragma unroll
    for (int q = 0; q < kRouteTok; ++q) acc[q] = gacc[q] = 0.f;

    const bool lane_is_expert = lane < E;
    for (int c = c_begin; c < c_end; ++c) {
        const int h0 = c * kWave;
        const int h = h0 + lane;
        float xv[kRouteTok];
#pragma unroll
        for (int q = 0; q < kRouteTok; ++q) {
            const int t = t0 + q;
            xv[q] = (t < T && h < d) ? load_f32(X, static_cast<size_t>(t) * d + h) : 0.f;
        }
        if (w_sg != nullptr) {
            const float g = h < d ? load_f32(w_sg, h) : 0.f;
#pragma unroll
            for (int q = 0; q < kRouteTok; ++q) gacc[q] += xv[q] * g;
        }
        const int n = min(kWave, d - h0);
#pragma unroll 8
        for (int i = 0; i < n; ++i) {
            const float wv =
                lane_is_expert ? load_f32(Wg, static_cast<size_t>(h0 + i) * E + lane) : 0.f;
#pragma unroll
            for (int q = 0; q < kRouteTok; ++q) acc[q] += __shfl(xv[q], i, kWave) * wv;
        }
    }
#pragma unroll
    for (int q = 0; q < kRouteTok; ++q) {
        part[wave][q][lane] = acc[q];
        if (w_sg != nullptr) {
            const float g = wave_sum(gacc[q]);
            if (lane == 0) gpart[wave][q] = g;
        }
    }
    __syncthreads();

    // wave q finishes token t0 + q
    for (int q = wave; q < kRouteTok; q += kRouteWaves) {
        const int t = t0 + q;
        if (t >= T) continue;
        float logit = 0.f;
#pragma unroll
        for (int w = 0; w < kRouteWaves; ++w) logit += part[w][q][lane];
        if (bias != nullptr && lane_is_expert) logit += bias[lane];
        if (!lane_is_expert) logit = -INFINITY;
        const float m = wave_max(logit);
        const float p = lane_is_expert ? expf(logit - m) : 0.f;
        const float den = wave_sum(p);
        const float s = p / den;
        if (scores != nullptr && lane_is_expert) scores[static_cast<size_t>(t) * E + lane] = s;
        wave_topk_store(s, lane_is_expert, K, topk_ids + static_cast<size_t>(t) * K,
                        topk_s + static_cast<size_t>(t) * K);
        if (w_sg != nullptr && lane == 0) {
            float g = 0.f;
#pragma unroll
            for (int w = 0; w < kRouteWaves; ++w) g += gpart[w][q];
            sgate[t] = 1.f / (1.f + expf(-g));
        }
    }
}

// ---------------------------------------------------------------------------
// bf16 fast path: the gate GEMM on the matrix cores.  A workgroup of 16 waves
// owns 16 tokens; the waves split the hidden dimension into slices of 32-wide
// steps, each wave running v_mfma_f32_16x16x32_bf16 on its slice with the A
// operand read straight from X (64 contiguous bytes per token and step) and the
// B operand from the gate matrix re-tiled by pack_gate_kernel (one 16-byte load
// per lane).  The partial logits meet in LDS in a fixed order, then one wave
// per token does the softmax and the Top-K with one lane per expert.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kRmTok = 16;
// 16 waves per workgroup: a workgroup is a chain of dependent steps (loads, reduction,
// softmax, Top-K) and at most a few workgroups run per compute unit, so a wave's share of
// the hidden dimension should be one batch of loads and a wave should finish one token
constexpr int kRmWaves = 16;

template <bool GATE>
__global__ __launch_bounds__(kRmWaves* kWave) void route_mfma_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ Gp, const float* __restrict__ bias,
    int T, int d, int E, int K, float* __restrict__ scores, int32_t* __restrict__ topk_ids,
    float* __restrict__ topk_s, float* __restrict__ sgate) {
    constexpr int NB = GATE ? kGateBlocks : kGateBlocks - 1;   // 16-column blocks
    __shared__ float red[kRmWaves][NB][4][kWave];

    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int t0 = blockIdx.x * kRmTok;
    const int KB = d / 32;
    const int per_wave = (KB + kRmWaves - 1) / kRmWaves;
    const int s0 = min(KB, wave * per_wave), s1 = min(KB, s0 + per_wave);

    const int m = lane % 16, kg = lane / 16;
    const bool a_ok = t0 + m < T;
    const bf16x8* ap =
        reinterpret_cast<const bf16x8*>(X + static_cast<size_t>(a_ok ? t0 + m : 0) * d) + kg;
    const bf16x8* bp = reinterpret_cast<const bf16x8*>(Gp) + lane;

    f32x4 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bf16x8 zero = {0};
    constexpr int U = 4;
    int s = s0;
    for (; s + U <= s1; s += U) {
        bf16x8 av[U], bv[U][NB];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            av[u] = a_ok ? ap[(s + u) * 4] : zero;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                bv[u][nb] = bp[(static_cast<size_t>(nb) * KB + s + u) * kWave];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u], bv[u][nb], acc[nb], 0, 0, 0);
    }
    for (; s < s1; ++s) {
        const bf16x8 av = a_ok ? ap[s * 4] : zero;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const bf16x8 bv = bp[(static_cast<size_t>(nb) * KB + s) * kWave];
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc[nb], 0, 0, 0);
        }
    }
    // accumulator register r of lane l holds C[4*(l/16) + r][l%16]
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][nb][r][lane] = acc[nb][r];
    __syncthreads();

    const bool lane_is_expert = lane < E;
    for (int q = wave; q < kRmTok; q += kRmWaves) {
        const int t = t0 + q;
        if (t >= T) continue;
        const int r = q % 4, lsrc = 16 * (q / 4);
        float logit = 0.f;
#pragma unroll
        for (int w = 0; w < kRmWaves; ++w) logit += red[w][lane / 16][r][lsrc + lane % 16];
        if (bias != nullptr && lane_is_expert) logit += bias[lane];
        if (!lane_is_expert) logit = -INFINITY;
        const float mx = wave_max(logit);
        const float p = lane_is_expert ? expf(logit - mx) : 0.f;
        const float den = wave_sum(p);
        const float sc = p / den;
        if (scores != nullptr && lane_is_expert) scores[static_cast<size_t>(t) * E + lane] = sc;
        wave_topk_store(sc, lane_is_expert, K, topk_ids + static_cast<size_t>(t) * K,
                        topk_s + static_cast<size_t>(t) * K);
        if (GATE && lane == 0) {
            float g = 0.f;
#pragma unroll
            for (int w = 0; w < kRmWaves; ++w) g += red[w][NB - 1][r][lsrc];
            sgate[t] = 1.f / (1.f + expf(-g));
        }
    }
}

// Re-tiles the gate matrix Wg [d,E] (and, as column 64, the shared expert's
// gate vector w_sg [d]) into the B-operand order of v_mfma_f32_16x16x32_bf16:
// fragment (nb, s) = 64 lanes x 8 values, lane l holding
//   G[32 s + 8 (l/16) + i][16 nb + l%16],  i = 0..7,
// with G's columns E..63 and 65..79 zero.  Layout: [nb][s][lane][8].
__global__ __launch_bounds__(256) void pack_gate_kernel(const bf16_t* __restrict__ Wg,
                                                        const bf16_t* __restrict__ w_sg, int d,
                                                        int E, bf16_t* __restrict__ out) {
    const int KB = d / 32;
    const int total = kGateBlocks * KB * kWave;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int l = idx % kWave, s = (idx / kWave) % KB, nb = idx / (kWave * KB);
    const int n = 16 * nb + l % 16, k0 = 32 * s + 8 * (l / 16);
    bf16_t* dst = out + static_cast<size_t>(idx) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        bf16_t v = 0;
        if (n < E)
            v = Wg[static_cast<size_t>(k0 + i) * E + n];
        else if (n == 64 && w_sg != nullptr)
            v = w_sg[k0 + i];
        dst[i] = v;
    }
}

// Candidates from caller-supplied scores: one wave per token.
__global__ __launch_bounds__(256) void topk_from_scores_kernel(
    const float* __restrict__ scores, int T, int E, int K, int32_t* __restrict__ topk_ids,
    float* __restrict__ topk_s) {
    const int lane = lane_id();
    const int t = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const bool valid = lane < E;
    const float s = valid ? scores[static_cast<size_t>(t) * E + lane] : 0.f;
    wave_topk_store(s, valid, K, topk_ids + static_cast<size_t>(t) * K,
                    topk_s + static_cast<size_t>(t) * K);
}

hipError_t launch_route(int dtype, const void* X, const void* Wg, const float* bias,
                        const void* w_sg, int T, int d, int E, int K, float* scores,
                        int32_t* topk_ids, float* topk_s, float* sgate, hipStream_t stream) {
    const dim3 grid((T + kRouteTok - 1) / kRouteTok), block(kRouteWaves * kWave);
    if (dtype == 0) {
        hipLaunchKernelGGL(route_kernel<float>, grid, block, 0, stream,
                           static_cast<const float*>(X), static_cast<const float*>(Wg), bias,
                           static_cast<const float*>(w_sg), T, d, E, K, scores, topk_ids, topk_s,
                           sgate);
    } else {
        hipLaunchKernelGGL(route_kernel<bf16_t>, grid, block, 0, stream,
                           static_cast<const bf16_t*>(X), static_cast<const bf16_t*>(Wg), bias,
                           static_cast<const bf16_t*>(w_sg), T, d, E, K, scores, topk_ids,
                           topk_s, sgate);
    }
    return hipGetLastError();
}

hipError_t launch_route_mfma(const void* X, const void* gate_packed, const float* bias,
                             bool with_gate, int T, int d, int E, int K, float* scores,
                             int32_t* topk_ids, float* topk_s, float* sgate,
                             hipStream_t stream) {
    const dim3 grid((T + kRmTok - 1) / kRmTok);
    const bf16_t* Xb = static_cast<const bf16_t*>(X);
    const bf16_t* Gp = static_cast<const bf16_t*>(gate_packed);
    const dim3 block(kRmWaves * kWave);
    if (with_gate)
        hipLaunchKernelGGL(route_mfma_kernel<true>, grid, block, 0, stream, Xb, Gp, bias, T, d, E,
                           K, scores, topk_ids, topk_s, sgate);
    else
        hipLaunchKernelGGL(route_mfma_kernel<false>, grid, block, 0, stream, Xb, Gp, bias, T, d, E,
                           K, scores, topk_ids, topk_s, sgate);
    return hipGetLastError();
}

hipError_t launch_pack_gate(const void* Wg, const void* w_sg, int d, int E, void* out,
                            hipStream_t stream) {
    const int total = kGateBlocks * (d / 32) * kWave;
    hipLaunchKernelGGL(pack_gate_kernel, dim3((total + 255) / 256), dim3(256), 0, stream,
                       static_cast<const bf16_t*>(Wg), static_cast<const bf16_t*>(w_sg), d, E,
                       static_cast<bf16_t*>(out));
    return hipGetLastError();
}

hipError_t launch_topk_from_scores(const float* scores, int T, int E, int K, int32_t* topk_ids,
                                   float* topk_s, hipStream_t stream) {
    const int waves = 4;
    const dim3 grid((T + waves - 1) / waves), block(waves * kWave);
    hipLaunchKernelGGL(topk_from_scores_kernel, grid, block, 0, stream, scores, T, E, K, topk_ids,
                       topk_s);
    return hipGetLastError();
}

}  // namespace allocmoe
