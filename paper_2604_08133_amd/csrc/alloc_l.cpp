// Alloc-L's sensitivity-guided layer-wise allocation (Section 3.2, Eqs. (3)-(5)):
// the grouped-knapsack dynamic programme DP[i][b] = min_k DP[i-1][b-k] + S[i][k]
// over the L layers and budgets 0..min(B, L*K_orig), answer at the best b <= B,
// allocation recovered by backtracking.  Host code: the paper runs this step
// offline; its result (K_l per layer) is what the layer calls take as budgets.
#include "../../include/allocmoe.h"

#include <algorithm>
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

// Heuristic layer-level schedules the paper compares Alloc-L with (appendix
// "Implementation Details of Baselines", layer-level baseline): Ascending grows the
// per-layer allocation with depth, Descending is its mirror image.
namespace {

// steps 1-2 of the description: rounded linear interpolation from lo (first layer) to
// hi (last layer), then one pass in each direction that leaves the vector
// non-decreasing with steps of at most one
void ramp(std::vector<int>& K, int lo, int hi) {
    const int L = static_cast<int>(K.size());
    for (int i = 0; i < L; ++i)
        K[i] = L == 1 ? lo
                      : static_cast<int>(std::floor(lo + static_cast<double>(hi - lo) * i / (L - 1) + 0.5));
    for (int i = 1; i < L; ++i) K[i] = std::min(std::max(K[i], K[i - 1]), K[i - 1] + 1);
    for (int i = L - 2; i >= 0; --i) K[i] = std::max(std::min(K[i], K[i + 1]), K[i + 1] - 1);
}

// step 3: sweeps over the internal layers, shallow to deep, each moving by one unit
// towards the budget where the vector stays non-decreasing, inside [lo, hi] and with
// steps of at most one.  Returns the sum reached (== B on success).
int64_t settle(std::vector<int>& K, int lo, int hi, int64_t B) {
    const int L = static_cast<int>(K.size());
    int64_t total = 0;
    for (int v : K) total += v;
    bool moved = true;
    while (total != B && moved) {
        moved = false;
        for (int i = 1; i + 1 < L && total != B; ++i) {
            if (total < B) {
                const int v = K[i] + 1;
                if (v <= hi && v <= K[i + 1] && v - K[i - 1] <= 1) {
                    K[i] = v;
                    ++total;
                    moved = true;
                }
            } else {
                const int v = K[i] - 1;
                if (v >= lo && v >= K[i - 1] && K[i + 1] - v <= 1) {
                    K[i] = v;
                    --total;
                    moved = true;
                }
            }
        }
    }
    return total;
}

}  // namespace

extern "C" allocmoe_status allocmoe_layer_schedule(allocmoe_schedule kind, int32_t L,
                                                   int32_t K_orig, int64_t B, int32_t* K_out) {
    if (K_out == nullptr || L < 1 || K_orig < 1) return ALLOCMOE_EINVAL;
    if (kind != ALLOCMOE_SCHEDULE_ASCENDING && kind != ALLOCMOE_SCHEDULE_DESCENDING)
        return ALLOCMOE_EINVAL;
    if (B < L || B > static_cast<int64_t>(L) * K_orig) return ALLOCMOE_EBUDGET;
    std::vector<int> K(static_cast<size_t>(L));
    bool found = false;
    if (L == 1) {
        K[0] = static_cast<int>(B);
        found = true;
    }
    // step 4: K_min = 1, K_max = K_orig; a budget above their reach raises K_min, one
    // below it lowers K_max
    for (int lo = 1, hi = K_orig; !found && lo <= hi;) {
        ramp(K, lo, hi);
        const int64_t total = settle(K, lo, hi, B);
        if (total == B)
            found = true;
        else if (total < B)
            ++lo;
        else
            --hi;
    }
    if (!found) return ALLOCMOE_EINVAL;   // not reached for L <= B <= L * K_orig
    for (int i = 0; i < L; ++i)
        K_out[i] = kind == ALLOCMOE_SCHEDULE_ASCENDING ? K[i] : K[L - 1 - i];
    return ALLOCMOE_OK;
}
