// Routing analytics of one layer's budgeted routing (Section 5, "Analysis of
// Expert Load Balance": expert loads under the original and the budgeted
// routing, Spearman rank correlation, normalised-entropy change and
// Jensen-Shannon divergence of the score-weighted load distributions; "Analysis
// of Budget Allocation": correlation between a token's routing entropy and the
// number of experts it keeps).
//
// "Original" routing keeps all K candidates of a token, budgeted routing the
// first keep_count[t].  No floating-point atomics: every sum has a fixed order,
// and both rank correlations are formed from exact integer sums of doubled
// average ranks (2 * rank = 2 * #smaller + #equal + 1).
#include "common.hpp"
#include "kernels.hpp"

namespace allocmoe {

namespace {

constexpr int kStatThreads = 256;

// H_t = -sum_e s ln s, one wave per token, lane = expert
__global__ __launch_bounds__(kStatThreads) void token_entropy_kernel(
    const float* __restrict__ scores, int T, int E, float* __restrict__ H) {
    const int lane = lane_id();
    const int t = blockIdx.x * (kStatThreads / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const float s = lane < E ? scores[static_cast<size_t>(t) * E + lane] : 0.f;
    const float term = s > 0.f ? -s * logf(s) : 0.f;
    const float h = wave_sum(term);
    if (lane == 0) H[t] = h;
}

// one workgroup per expert: counts and score sums of its candidate pairs and of
// its kept pairs; thread-strided partial sums, then a fixed-order tree
__global__ __launch_bounds__(kStatThreads) void expert_load_kernel(
    const int32_t* __restrict__ topk_ids, const float* __restrict__ topk_s,
    const int32_t* __restrict__ keep_count, int T, int K, int32_t* __restrict__ load_orig,
    int32_t* __restrict__ load_kept, float* __restrict__ wload_orig,
    float* __restrict__ wload_kept) {
    __shared__ int32_t cnt[2][kStatThreads];
    __shared__ float wsum[2][kStatThreads];
    const int e = blockIdx.x, tid = threadIdx.x;
    int co = 0, ck = 0;
    float wo = 0.f, wk = 0.f;
    for (int t = tid; t < T; t += kStatThreads) {
        const int kt = keep_count[t];
        for (int j = 0; j < K; ++j) {
            if (topk_ids[static_cast<size_t>(t) * K + j] != e) continue;
            const float s = topk_s[static_cast<size_t>(t) * K + j];
            ++co;
            wo += s;
            if (j < kt) {
                ++ck;
                wk += s;
            }
        }
    }
    cnt[0][tid] = co;
    cnt[1][tid] = ck;
    wsum[0][tid] = wo;
    wsum[1][tid] = wk;
    __syncthreads();
    for (int half = kStatThreads / 2; half >= 1; half >>= 1) {
        if (tid < half) {
            cnt[0][tid] += cnt[0][tid + half];
            cnt[1][tid] += cnt[1][tid + half];
            wsum[0][tid] += wsum[0][tid + half];
            wsum[1][tid] += wsum[1][tid + half];
        }
        __syncthreads();
    }
    if (tid == 0) {
        load_orig[e] = cnt[0][0];
        load_kept[e] = cnt[1][0];
        wload_orig[e] = wsum[0][0];
        wload_kept[e] = wsum[1][0];
    }
}

// doubled average rank of every token's entropy among all T entropies
__global__ __launch_bounds__(kStatThreads) void entropy_rank_kernel(const float* __restrict__ H,
                                                                    int T,
                                                                    int32_t* __restrict__ rank2) {
    __shared__ float tile[kStatThreads];
    const int t = blockIdx.x * kStatThreads + threadIdx.x;
    const float mine = t < T ? H[t] : 0.f;
    int less = 0, equal = 0;
    for (int base = 0; base < T; base += kStatThreads) {
        const int u = base + threadIdx.x;
        __syncthreads();
        tile[threadIdx.x] = u < T ? H[u] : 0.f;
        __syncthreads();
        const int n = min(kStatThreads, T - base);
        for (int i = 0; i < n; ++i) {
            const float v = tile[i];
            less += v < mine ? 1 : 0;
            equal += v == mine ? 1 : 0;
        }
    }
    if (t < T) rank2[t] = 2 * less + equal + 1;
}

__device__ __forceinline__ long long block_sum_i64(long long v, long long* buf) {
    const int tid = threadIdx.x;
    __syncthreads();
    buf[tid] = v;
    __syncthreads();
    for (int half = kStatThreads / 2; half >= 1; half >>= 1) {
        if (tid < half) buf[tid] += buf[tid + half];
        __syncthreads();
    }
    return buf[0];
}

// Pearson correlation of two rank vectors from exact integer sums (doubled ranks)
__device__ __forceinline__ float rank_correlation(long long n, long long sa, long long sb,
                                                  long long saa, long long sbb, long long sab) {
    const double va = static_cast<double>(n) * static_cast<double>(saa) -
                      static_cast<double>(sa) * static_cast<double>(sa);
    const double vb = static_cast<double>(n) * static_cast<double>(sbb) -
                      static_cast<double>(sb) * static_cast<double>(sb);
    const double cov = static_cast<double>(n) * static_cast<double>(sab) -
                       static_cast<double>(sa) * static_cast<double>(sb);
    if (va <= 0.0 || vb <= 0.0) return 0.f;   // one side constant
    return static_cast<float>(cov / sqrt(va * vb));
}

// one workgroup: the five summary numbers
__global__ __launch_bounds__(kStatThreads) void routing_metrics_kernel(
    const int32_t* __restrict__ load_orig, const int32_t* __restrict__ load_kept,
    const float* __restrict__ wload_orig, const float* __restrict__ wload_kept,
    const int32_t* __restrict__ keep_count, const int32_t* __restrict__ entropy_rank2, int T,
    int E, int K, float* __restrict__ metrics) {
    __shared__ long long buf[kStatThreads];
    __shared__ int32_t k_hist[64];
    const int tid = threadIdx.x, lane = lane_id();

    // ---- expert side, first wave, lane = expert
    if (tid < kWave) {
        const bool valid = lane < E;
        const int lo = valid ? load_orig[lane] : 0, lk = valid ? load_kept[lane] : 0;
        int ro = 1, rk = 1;   // doubled average ranks among the E loads
        for (int o = 0; o < E; ++o) {
            const int oo = __shfl(lo, o, kWave), ok = __shfl(lk, o, kWave);
            ro += oo < lo ? 2 : (oo == lo ? 1 : 0);
            rk += ok < lk ? 2 : (ok == lk ? 1 : 0);
        }
        auto isum = [&](long long v) {
#pragma unroll
            for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, kWave);
            return v;
        };
        const long long a = valid ? ro : 0, b = valid ? rk : 0;
        const float rho = rank_correlation(E, isum(a), isum(b), isum(a * a), isum(b * b), isum(a * b));
        // weighted load distributions
        const float wo = valid ? wload_orig[lane] : 0.f, wk = valid ? wload_kept[lane] : 0.f;
        const float so = wave_sum(wo), sk = wave_sum(wk);
        const float p = so > 0.f ? wo / so : 0.f, q = sk > 0.f ? wk / sk : 0.f;
        const float norm = E > 1 ? 1.f / logf(static_cast<float>(E)) : 0.f;
        const float ho = wave_sum(p > 0.f ? -p * logf(p) : 0.f) * norm;
        const float hk = wave_sum(q > 0.f ? -q * logf(q) : 0.f) * norm;
        const float m = 0.5f * (p + q);
        const float js = 0.5f * wave_sum((p > 0.f ? p * logf(p / m) : 0.f) +
                                         (q > 0.f ? q * logf(q / m) : 0.f));
        if (lane == 0) {
            metrics[0] = rho;
            metrics[1] = ho;
            metrics[2] = hk;
            metrics[3] = js;
        }
    }

    // ---- token side: doubled ranks of keep_count from its histogram (values 0..K)
    if (tid < 64) k_hist[tid] = 0;
    __syncthreads();
    for (int t = tid; t < T; t += kStatThreads) atomicAdd(&k_hist[keep_count[t]], 1);   // integers
    __syncthreads();
    long long sa = 0, sb = 0, saa = 0, sbb = 0, sab = 0;
    for (int t = tid; t < T; t += kStatThreads) {
        const int v = keep_count[t];
        int below = 0;
        for (int u = 0; u < v; ++u) below += k_hist[u];
        const long long b = 2ll * below + k_hist[v] + 1, a = entropy_rank2[t];
        sa += a;
        sb += b;
        saa += a * a;
        sbb += b * b;
        sab += a * b;
    }
    sa = block_sum_i64(sa, buf);
    sb = block_sum_i64(sb, buf);
    saa = block_sum_i64(saa, buf);
    sbb = block_sum_i64(sbb, buf);
    sab = block_sum_i64(sab, buf);
    if (tid == 0) metrics[4] = rank_correlation(T, sa, sb, saa, sbb, sab);
    (void)K;
}

}  // namespace

hipError_t launch_routing_stats(const float* scores, const int32_t* topk_ids, const float* topk_s,
                                const int32_t* keep_count, int T, int E, int K,
                                int32_t* load_orig, int32_t* load_kept, float* wload_orig,
                                float* wload_kept, float* token_entropy, int32_t* entropy_rank2,
                                float* metrics, hipStream_t stream) {
    const int tokens_per_wg = kStatThreads / kWave;
    hipLaunchKernelGGL(token_entropy_kernel, dim3((T + tokens_per_wg - 1) / tokens_per_wg),
                       dim3(kStatThreads), 0, stream, scores, T, E, token_entropy);
    hipLaunchKernelGGL(expert_load_kernel, dim3(E), dim3(kStatThreads), 0, stream, topk_ids,
                       topk_s, keep_count, T, K, load_orig, load_kept, wload_orig, wload_kept);
    hipLaunchKernelGGL(entropy_rank_kernel, dim3((T + kStatThreads - 1) / kStatThreads),
                       dim3(kStatThreads), 0, stream, token_entropy, T, entropy_rank2);
    hipLaunchKernelGGL(routing_metrics_kernel, dim3(1), dim3(kStatThreads), 0, stream, load_orig,
                       load_kept, wload_orig, wload_kept, keep_count, entropy_rank2, T, E, K,
                       metrics);
    return hipGetLastError();
}

}  // namespace allocmoe
