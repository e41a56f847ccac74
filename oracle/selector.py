"""Layer selection (Sec. 4.3 "Layer Selection Algorithm", Problem 4.5, App. D) -- oracle, test infrastructure only.

Three plain pieces, float64 throughout:
  * hill_alpha: the Hill estimator of the power-law tail exponent on the largest chi eigenvalues;
  * benefits: nu_i = (alpha_max - alpha_i) / (alpha_max - alpha_min) * P_i / sum_j P_j;
  * Problem 4.5 itself, by exhaustive search over what the integer program allows (every verifier takes no
    interval or one contiguous interval within its budget, intervals pairwise disjoint), in two variants:
    `best_assignment` (any verifier anywhere: the integer program as printed) and `best_ordered_assignment`
    (the intervals of verifiers 1..M appear left to right, which is what the recursion of App. D enumerates);
    and the recursion of App. D written out naively, O(M L^2).

Reading: the printed recursion inherits only DP[k, i-1]; with DP[k, 0] = 0 that can never carry what verifiers
1..k-1 reach when verifier k stays idle, which Case 1 of the proof assumes it does.  The recursion here (and in the
library) also takes DP[k-1, i].
"""
import itertools
import math


def hill_alpha(eigenvalues, chi):
    """alpha_hat = 1 + chi / sum_{r=1..chi} ln(Lambda_{d-r+1} / Lambda_{d-chi}), eigenvalues ascending, 1-based."""
    lam = sorted(float(x) for x in eigenvalues)
    d = len(lam)
    if not (1 <= chi < d):
        raise ValueError("chi must satisfy 1 <= chi < d")
    base = lam[d - chi - 1]                                   # Lambda_{d - chi}
    total = sum(math.log(lam[d - r] / base) for r in range(1, chi + 1))
    return 1.0 + chi / total


def benefits(alphas, params):
    amax, amin = max(alphas), min(alphas)
    total = float(sum(params))
    if amax == amin:
        return [0.0 for _ in alphas]
    return [(amax - a) / (amax - amin) * (p / total) for a, p in zip(alphas, params)]


def _intervals(L):
    yield None
    for s in range(L):
        for e in range(s, L):
            yield (s, e)


def _feasible(choice, nu, phi, beta):
    used = set()
    value = 0.0
    for iv, b in zip(choice, beta):
        if iv is None:
            continue
        s, e = iv
        if sum(phi[s : e + 1]) > b:
            return None
        span = set(range(s, e + 1))
        if used & span:
            return None
        used |= span
        value += sum(nu[s : e + 1])
    return value


def best_assignment(nu, phi, beta):
    """The integer program of Problem 4.5 by brute force (tiny instances only)."""
    best = 0.0
    for choice in itertools.product(list(_intervals(len(nu))), repeat=len(beta)):
        v = _feasible(choice, nu, phi, beta)
        if v is not None and v > best:
            best = v
    return best


def best_ordered_assignment(nu, phi, beta):
    """Same, with the intervals of verifiers 1..M in left-to-right order."""
    best = 0.0
    for choice in itertools.product(list(_intervals(len(nu))), repeat=len(beta)):
        last = -1
        ordered = True
        for iv in choice:
            if iv is not None:
                if iv[0] <= last:
                    ordered = False
                    break
                last = iv[1]
        if not ordered:
            continue
        v = _feasible(choice, nu, phi, beta)
        if v is not None and v > best:
            best = v
    return best


def dp_naive(nu, phi, beta):
    """DP[k][i] of App. D with every start scanned; returns the table (k = 0..M, i = 0..L)."""
    L, M = len(nu), len(beta)
    V = [0.0] * (L + 1)
    C = [0.0] * (L + 1)
    for i in range(L):
        V[i + 1] = V[i] + nu[i]
        C[i + 1] = C[i] + phi[i]
    DP = [[0.0] * (L + 1) for _ in range(M + 1)]
    for k in range(1, M + 1):
        for i in range(1, L + 1):
            best = max(DP[k][i - 1], DP[k - 1][i])
            for s in range(1, i + 1):
                if C[i] - C[s - 1] <= beta[k - 1]:
                    best = max(best, V[i] - V[s - 1] + DP[k - 1][s - 1])
            DP[k][i] = best
    return DP
