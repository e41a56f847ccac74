/*
 * Layer selection on the host (Sec. 4.3; Problem 4.5; App. D): the verifier decides which layers to open.
 * Plain C++, float64, no GPU.
 *
 * select_layers runs the recursion of App. D,
 *     DP[k, i] = max{ DP[k, i-1], DP[k-1, i], max_{s <= i, C[i] - C[s-1] <= beta_k} V[i] - V[s-1] + DP[k-1, s-1] },
 * with prefix sums V, C of benefits and costs.  For fixed k the feasible starts form a window that only moves
 * right (costs are positive), and the inner maximum is V[i] plus the maximum of F(s) = DP[k-1, s-1] - V[s-1] over
 * that window: a deque of candidate starts with F strictly decreasing from front to back gives it in O(1)
 * amortised, O(M L) altogether.  DP[k-1, i] (verifier k idle) is not in the printed recursion, whose boundary
 * DP[k, 0] = 0 cannot carry it; the proof's first case needs it.  The recursion places the intervals of
 * verifiers 1..M from left to right.
 */
#pragma once
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include <algorithm>
#include <deque>
#include <vector>

namespace tc {
namespace selector {

/* 1 + chi / sum_{r=1..chi} ln(Lambda_{d-r+1} / Lambda_{d-chi}); eigenvalues in any order (sorted here) */
inline bool hill_alpha(const double* eig, size_t d, size_t chi, double* out) {
    if (!eig || !out || chi < 1 || chi >= d) return false;
    std::vector<double> lam(eig, eig + d);
    std::sort(lam.begin(), lam.end());
    double base = lam[d - chi - 1];
    if (!(base > 0.0)) return false;
    double total = 0.0;
    for (size_t r = 1; r <= chi; ++r) total += log(lam[d - r] / base);
    if (!(total > 0.0)) return false;
    *out = 1.0 + (double)chi / total;
    return true;
}

inline void benefits(const double* alpha, const double* params, size_t L, double* nu) {
    double amax = alpha[0], amin = alpha[0], total = 0.0;
    for (size_t i = 0; i < L; ++i) {
        amax = std::max(amax, alpha[i]);
        amin = std::min(amin, alpha[i]);
        total += params[i];
    }
    for (size_t i = 0; i < L; ++i) nu[i] = amax == amin ? 0.0 : (amax - alpha[i]) / (amax - amin) * (params[i] / total);
}

/* value = DP[M, L]; start[k], end[k] = the interval of verifier k (0-based, inclusive) or -1, -1 */
inline double select_layers(size_t L, const double* nu, const double* phi, size_t M, const double* beta, int64_t* start,
                            int64_t* end) {
    std::vector<double> V(L + 1, 0.0), C(L + 1, 0.0);
    for (size_t i = 0; i < L; ++i) {
        V[i + 1] = V[i] + nu[i];
        C[i + 1] = C[i] + phi[i];
    }
    std::vector<double> prev(L + 1, 0.0), cur(L + 1, 0.0);
    /* how DP[k, i] was reached: -1 = DP[k, i-1], -2 = DP[k-1, i], s >= 1 = interval [s, i] */
    std::vector<std::vector<int32_t>> how(M, std::vector<int32_t>(L + 1, -1));
    for (size_t k = 1; k <= M; ++k) {
        std::deque<size_t> window;               /* starts s, F strictly decreasing front to back */
        cur[0] = 0.0;
        for (size_t i = 1; i <= L; ++i) {
            double fi = prev[i - 1] - V[i - 1];  /* F(i): the start s = i becomes available */
            while (!window.empty() && prev[window.back() - 1] - V[window.back() - 1] <= fi) window.pop_back();
            window.push_back(i);
            while (!window.empty() && C[i] - C[window.front() - 1] > beta[k - 1]) window.pop_front();
            double best = cur[i - 1];
            int32_t via = -1;
            if (prev[i] > best) { best = prev[i]; via = -2; }
            if (!window.empty()) {
                size_t s = window.front();
                double cand = V[i] + (prev[s - 1] - V[s - 1]);
                if (cand > best) { best = cand; via = (int32_t)s; }
            }
            cur[i] = best;
            how[k - 1][i] = via;
        }
        prev.swap(cur);
    }
    double value = prev[L];
    for (size_t k = 0; k < M; ++k) start[k] = end[k] = -1;
    size_t k = M, i = L;
    while (k >= 1 && i >= 1) {
        int32_t via = how[k - 1][i];
        if (via == -1) {
            --i;
        } else if (via == -2) {
            --k;
        } else {
            start[k - 1] = via - 1;
            end[k - 1] = (int64_t)i - 1;
            i = (size_t)via - 1;
            --k;
        }
    }
    return value;
}

}  // namespace selector
}  // namespace tc
