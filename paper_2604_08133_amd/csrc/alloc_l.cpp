// Alloc-L's sensitivity-guided layer-wise allocation (Section 3.2, Eqs. (3)-(5)):
// the grouped-knapsack dynamic programme DP[i][b] = min_k DP[i-1][b-k] + S[i][k]
// over the L layers and budgets 0..min(B, L*K_orig), answer at the best b <= B,
// allocation recovered by backtracking.  Host code: the paper runs this step
// offline; its result (K_l per layer) is what the layer calls take as budgets.
#include "../../include/allocmoe.h"

#include <cmath>
#include <limits>
#include <vector>

extern "C" allocmoe_status allocmoe_alloc_l(const double* S, int32_t L, int32_t K_orig,
                                            int64_t B, int32_t* K_out, double* cost_out) {
    if (S == nullptr || K_out == nullptr || L < 1 || K_orig < 1) return ALLOCMOE_EINVAL;
    if (static_cast<int64_t>(L) * K_orig > (int64_t{1} << 24)) return ALLOCMOE_ESHAPE;
    if (B < L) return ALLOCMOE_EBUDGET;   // Eq. (5): every layer keeps at least one expert
    for (int64_t i = 0; i < static_cast<int64_t>(L) * K_orig; ++i)
        if (std::isnan(S[i])) return ALLOCMOE_EINVAL;
    const int top = static_cast<int>(std::min<int64_t>(B, static_cast<int64_t>(L) * K_orig));
    const double inf = std::numeric_limits<double>::infinity();
    const size_t width = static_cast<size_t>(top) + 1;
    // rows -1 .. L-1 of the table, row -1 first
    std::vector<double> dp((static_cast<size_t>(L) + 1) * width, inf);
    dp[0] = 0.0;
    for (int i = 0; i < L; ++i) {
        const double* prev = dp.data() + static_cast<size_t>(i) * width;
        double* cur = dp.data() + static_cast<size_t>(i + 1) * width;
        const double* s = S + static_cast<size_t>(i) * K_orig;
        // after layer i at least i+1 and at most (i+1)*K_orig units are spent
        const int b_hi = std::min<int64_t>(top, static_cast<int64_t>(i + 1) * K_orig);
        for (int b = i + 1; b <= b_hi; ++b) {
            double best = inf;
            const int k_hi = std::min(K_orig, b);
            for (int k = 1; k <= k_hi; ++k) {
                const double c = prev[b - k] + s[k - 1];
                if (c < best) best = c;
            }
            cur[b] = best;
        }
    }
    // the cheapest total; of equal totals the smaller spend
    const double* last = dp.data() + static_cast<size_t>(L) * width;
    int best_b = -1;
    for (int b = 0; b <= top; ++b)
        if (best_b < 0 || last[b] < last[best_b]) best_b = b;
    if (best_b < 0 || last[best_b] == inf) return ALLOCMOE_EINVAL;   // only with +inf entries in S
    // backtracking; of equal continuations the smaller K at the deeper layer
    int b = best_b;
    for (int i = L - 1; i >= 0; --i) {
        const double* prev = dp.data() + static_cast<size_t>(i) * width;
        const double* cur = dp.data() + static_cast<size_t>(i + 1) * width;
        const double* s = S + static_cast<size_t>(i) * K_orig;
        int pick = 0;
        for (int k = 1; k <= std::min(K_orig, b); ++k)
            if (prev[b - k] + s[k - 1] == cur[b]) {
                pick = k;
                break;
            }
        if (pick == 0) return ALLOCMOE_EINVAL;
        K_out[i] = pick;
        b -= pick;
    }
    if (cost_out != nullptr) *cost_out = last[best_b];
    return ALLOCMOE_OK;
}
