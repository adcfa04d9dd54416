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

// Sorted Top-K of N tokens' scores at once, lane = expert: larger score first, equal
// scores lower expert first.  K rounds of: the largest remaining key of the wave, the
// lowest lane that holds it stores its (expert, score) at the round's position and
// leaves.  (The N chains are independent; the compiler interleaves them.)
template <int N>
__device__ __forceinline__ void wave_topk_store_n(const float (&score)[N], bool valid, int K,
                                                  int32_t* const (&ids_row)[N],
                                                  float* const (&s_row)[N], const bool (&live)[N]) {
    const int lane = lane_id();
    // valid lanes: key >= 1 (scores are >= 0, so ordered_key has its top bit set)
    uint32_t key[N];
#pragma unroll
    for (int i = 0; i < N; ++i) key[i] = valid ? ordered_key(score[i]) : 0u;
    for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const uint32_t top = wave_max_u32(key[i]);
            const uint64_t holders = __ballot(key[i] == top);
            const int winner = __builtin_ctzll(holders);   // (holders != 0: every lane takes part)
            if (top != 0u && lane == winner) {
                if (live[i]) {
                    ids_row[i][k] = lane;
                    s_row[i][k] = score[i];
                }
                key[i] = 0u;
            }
        }
    }
}

__device__ __forceinline__ void wave_topk_store(float score, bool valid, int K,
                                                int32_t* __restrict__ ids_row,
                                                float* __restrict__ s_row) {
    const float sc[1] = {score};
    int32_t* const ids[1] = {ids_row};
    float* const ss[1] = {s_row};
    const bool live[1] = {true};
    wave_topk_store_n<1>(sc, valid, K, ids, ss, live);
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
// owns 16 MT tokens; the waves split the hidden dimension into slices of 32-wide
// steps, each wave running v_mfma_f32_16x16x32_bf16 on its slice with the A
// operand read straight from X (64 contiguous bytes per token and step) and the
// B operand from the gate matrix re-tiled by pack_gate_kernel (one 16-byte load
// per lane).  The partial logits meet in LDS in a fixed order, then one wave
// per token does the softmax and the Top-K with one lane per expert.
//
// A workgroup is bound by the bytes that cross its compute unit's vector load path
// (64 B per clock): the whole re-tiled gate matrix (262 KB, 327 KB with the shared
// gate's column) plus 4 KB per token, about 6 us at 16 tokens, whatever the token
// count.  Up to 4096 tokens that is one round of at most 256 workgroups.  Beyond,
// MT = 2: a wave multiplies every gate fragment it loads with two 16-token
// fragments, a workgroup owns 32 tokens and the launch stays one round up to 8192
// tokens.  Under the 128 registers a wave of a 16-wave workgroup gets, the loads then
// go out as two batches of two steps instead of one of four, which gives back most of
// what the halved gate traffic saves (8192 tokens: 22.7 instead of 25 us).  The partial
// sums of 16 waves x 2 token fragments would not fit the LDS at once: the upper eight
// waves hand theirs to the lower eight, which add their own and publish the sums.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kRmTok = 16;
// 16 waves per workgroup: a workgroup is a chain of dependent steps (loads, reduction,
// softmax, Top-K) and at most a few workgroups run per compute unit, so a wave's share of
// the hidden dimension should be one batch of loads and a wave should finish one token
constexpr int kRmWaves = 16;

template <bool GATE, int MT>
__global__ __launch_bounds__(kRmWaves* kWave) void route_mfma_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ Gp, const float* __restrict__ bias,
    int T, int d, int E, int K, float* __restrict__ scores, int32_t* __restrict__ topk_ids,
    float* __restrict__ topk_s, float* __restrict__ sgate) {
    static_assert(MT == 1 || MT == 2, "token fragments per wave");
    constexpr int NB = GATE ? kGateBlocks : kGateBlocks - 1;   // 16-column blocks
    constexpr int kSlots = MT == 1 ? kRmWaves : kRmWaves / 2;  // partial sums that meet in LDS
    __shared__ float red[kSlots][MT][NB][4][kWave];

    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int t0 = blockIdx.x * (kRmTok * MT);
    const int KB = d / 32;
    const int per_wave = (KB + kRmWaves - 1) / kRmWaves;
    const int s0 = min(KB, wave * per_wave), s1 = min(KB, s0 + per_wave);

    const int m = lane % 16, kg = lane / 16;
    bool a_ok[MT];
    const bf16x8* ap[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int t = t0 + kRmTok * mt + m;
        a_ok[mt] = t < T;
        ap[mt] = reinterpret_cast<const bf16x8*>(X + static_cast<size_t>(a_ok[mt] ? t : 0) * d) + kg;
    }
    const bf16x8* bp = reinterpret_cast<const bf16x8*>(Gp) + lane;

    f32x4 acc[MT][NB];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[mt][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bf16x8 zero = {0};
    constexpr int U = MT == 1 ? 4 : 2;   // steps per batch of loads (registers: 16 waves, 128 each)
    int s = s0;
    for (; s + U <= s1; s += U) {
        bf16x8 av[U][MT], bv[U][NB];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) av[u][mt] = a_ok[mt] ? ap[mt][(s + u) * 4] : zero;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                bv[u][nb] = bp[(static_cast<size_t>(nb) * KB + s + u) * kWave];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mt][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u][mt], bv[u][nb],
                                                                          acc[mt][nb], 0, 0, 0);
    }
    for (; s < s1; ++s) {
        bf16x8 av[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) av[mt] = a_ok[mt] ? ap[mt][s * 4] : zero;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const bf16x8 bv = bp[(static_cast<size_t>(nb) * KB + s) * kWave];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mt], bv, acc[mt][nb], 0, 0, 0);
        }
    }
    // accumulator register r of lane l holds C[4*(l/16) + r][l%16]
    if (MT == 1 || wave >= kSlots) {
        const int slot = MT == 1 ? wave : wave - kSlots;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int r = 0; r < 4; ++r) red[slot][mt][nb][r][lane] = acc[mt][nb][r];
    }
    __syncthreads();
    if (MT == 2) {
        if (wave < kSlots) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        red[wave][mt][nb][r][lane] = acc[mt][nb][r] + red[wave][mt][nb][r][lane];
        }
        __syncthreads();
    }

    // wave w finishes token w of every token fragment
    const bool lane_is_expert = lane < E;
    const int r = wave % 4, lsrc = 16 * (wave / 4);
    float sc[MT];
    bool live[MT];
    int32_t* ids_row[MT];
    float* s_row[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int t = t0 + kRmTok * mt + wave;
        live[mt] = t < T;
        const size_t tt = live[mt] ? t : 0;
        ids_row[mt] = topk_ids + tt * K;
        s_row[mt] = topk_s + tt * K;
        float logit = 0.f;
#pragma unroll
        for (int w = 0; w < kSlots; ++w) logit += red[w][mt][lane / 16][r][lsrc + lane % 16];
        if (bias != nullptr && lane_is_expert) logit += bias[lane];
        if (!lane_is_expert) logit = -INFINITY;
        const float mx = wave_max(logit);
        const float p = lane_is_expert ? expf(logit - mx) : 0.f;
        const float den = wave_sum(p);
        sc[mt] = p / den;
        if (live[mt] && scores != nullptr && lane_is_expert) scores[tt * E + lane] = sc[mt];
    }
    wave_topk_store_n<MT>(sc, lane_is_expert, K, ids_row, s_row, live);
    if (GATE && lane == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (!live[mt]) continue;
            float g = 0.f;
#pragma unroll
            for (int w = 0; w < kSlots; ++w) g += red[w][mt][NB - 1][r][lsrc];
            sgate[t0 + kRmTok * mt + wave] = 1.f / (1.f + expf(-g));
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
    const bf16_t* Xb = static_cast<const bf16_t*>(X);
    const bf16_t* Gp = static_cast<const bf16_t*>(gate_packed);
    const dim3 block(kRmWaves * kWave);
    // 32 tokens per workgroup where 16 would need more workgroups than compute units
    const bool wide = T > 256 * kRmTok;
    const int per_group = wide ? 2 * kRmTok : kRmTok;
    const dim3 grid((T + per_group - 1) / per_group);
#define ALLOCMOE_ROUTE_LAUNCH(gate, mt)                                                            \
    hipLaunchKernelGGL((route_mfma_kernel<gate, mt>), grid, block, 0, stream, Xb, Gp, bias, T, d,  \
                       E, K, scores, topk_ids, topk_s, sgate)
    if (with_gate && wide)
        ALLOCMOE_ROUTE_LAUNCH(true, 2);
    else if (with_gate)
        ALLOCMOE_ROUTE_LAUNCH(true, 1);
    else if (wide)
        ALLOCMOE_ROUTE_LAUNCH(false, 2);
    else
        ALLOCMOE_ROUTE_LAUNCH(false, 1);
#undef ALLOCMOE_ROUTE_LAUNCH
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
