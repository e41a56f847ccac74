"""Layer selection (Sec. 4.3, Problem 4.5, App. D): the oracle pinned to closed forms and to exhaustive search over
the integer program, the library's O(M L) dynamic program against the oracle.  CPU only."""
import math
import os
import random
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import __graft_entry__ as entry  # noqa: E402
import paper_2602_12630_amd as T  # noqa: E402
from oracle import selector as osel  # noqa: E402
from paper_2602_12630_amd import binding  # noqa: E402


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(T.library_path()):
        entry.build_hip()
    return T.load_library()


def test_hill_estimator_closed_forms(lib):
    # the chi largest eigenvalues all e^t times the (d - chi)-th: every log ratio is t, alpha = 1 + 1/t
    for t in (0.5, 2.0):
        eig = [0.1, 0.2, 1.0] + [math.exp(t)] * 4
        assert osel.hill_alpha(eig, 4) == pytest.approx(1 + 1 / t, rel=1e-14)
        assert binding.hill_alpha(eig, 4, lib) == pytest.approx(1 + 1 / t, rel=1e-14)
    # exact quantiles of a Pareto tail with density exponent alpha: the estimate approaches alpha as chi grows
    alpha, d, chi = 2.5, 20000, 2000
    eig = [(1 - (j + 0.5) / d) ** (-1 / (alpha - 1)) for j in range(d)]
    est = osel.hill_alpha(eig, chi)
    assert abs(est - alpha) < 0.05
    rng = random.Random(3)
    eig = [rng.paretovariate(1.7) for _ in range(500)]
    rng.shuffle(eig)
    assert binding.hill_alpha(eig, 50, lib) == pytest.approx(osel.hill_alpha(eig, 50), rel=1e-13)
    with pytest.raises(binding.TcError):
        binding.hill_alpha([1.0, 2.0], 2, lib)


def test_benefits(lib):
    assert osel.benefits([2.0, 3.0, 4.0], [1, 1, 2]) == [0.25, 0.125, 0.0]
    assert binding.layer_benefits([2.0, 3.0, 4.0], [1, 1, 2], lib) == [0.25, 0.125, 0.0]
    assert binding.layer_benefits([2.0, 2.0], [1, 3], lib) == [0.0, 0.0] == osel.benefits([2.0, 2.0], [1, 3])


def dp_as_printed(nu, phi, beta):
    """The recursion exactly as printed (no idle branch), for the counter-example below."""
    L, M = len(nu), len(beta)
    V, C = [0.0], [0.0]
    for a, b in zip(nu, phi):
        V.append(V[-1] + a)
        C.append(C[-1] + b)
    DP = [[0.0] * (L + 1) for _ in range(M + 1)]
    for k in range(1, M + 1):
        for i in range(1, L + 1):
            best = DP[k][i - 1]
            for s in range(1, i + 1):
                if C[i] - C[s - 1] <= beta[k - 1]:
                    best = max(best, V[i] - V[s - 1] + DP[k - 1][s - 1])
            DP[k][i] = best
    return DP[M][L]


def test_recursion_against_exhaustive_search():
    rng = random.Random(7)
    for _ in range(60):
        L, M = rng.randint(1, 5), rng.randint(1, 3)
        nu = [rng.randint(0, 9) / 4 for _ in range(L)]
        phi = [rng.randint(1, 5) for _ in range(L)]
        beta = [rng.randint(0, 9) for _ in range(M)]
        assert osel.dp_naive(nu, phi, beta)[M][L] == pytest.approx(osel.best_ordered_assignment(nu, phi, beta), abs=1e-12)
        same = [beta[0]] * M                     # equal budgets: the order of the verifiers does not matter
        assert osel.dp_naive(nu, phi, same)[M][L] == pytest.approx(osel.best_assignment(nu, phi, same), abs=1e-12)
    # the idle branch matters: a second verifier too poor for any layer must not erase what the first one reached
    nu, phi, beta = [1.0, 2.0], [1.0, 1.0], [2.0, 0.5]
    assert osel.best_assignment(nu, phi, beta) == 3.0 == osel.dp_naive(nu, phi, beta)[2][2]
    assert dp_as_printed(nu, phi, beta) == 0.0
    # unequal budgets: the left-to-right order of the verifiers can cost benefit against the integer program
    nu, phi, beta = [5.0, 5.0, 0.0, 1.0], [1.0, 1.0, 5.0, 1.0], [1.0, 2.0]
    assert osel.best_assignment(nu, phi, beta) == 11.0            # verifier 2 takes layers 1-2, verifier 1 layer 4
    assert osel.dp_naive(nu, phi, beta)[2][4] == 10.0 == osel.best_ordered_assignment(nu, phi, beta)


def check_solution(nu, phi, beta, value, intervals):
    last, total = -1, 0.0
    for k, iv in enumerate(intervals):
        if iv is None:
            continue
        s, e = iv
        assert last < s <= e < len(nu)
        assert sum(phi[s : e + 1]) <= beta[k] * (1 + 1e-12)
        total += sum(nu[s : e + 1])
        last = e
    assert total == pytest.approx(value, rel=1e-9, abs=1e-12)


def test_library_dynamic_program(lib):
    rng = random.Random(11)
    for _ in range(200):
        L, M = rng.randint(1, 12), rng.randint(1, 4)
        nu = [rng.random() for _ in range(L)]
        phi = [rng.random() + 0.05 for _ in range(L)]
        beta = [rng.random() * 3 for _ in range(M)]
        value, intervals = binding.select_layers(nu, phi, beta, lib)
        assert value == pytest.approx(osel.dp_naive(nu, phi, beta)[M][L], rel=1e-12, abs=1e-15)
        check_solution(nu, phi, beta, value, intervals)
    # integer data: exact equality, ties included
    for _ in range(100):
        L, M = rng.randint(1, 10), rng.randint(1, 3)
        nu = [float(rng.randint(0, 3)) for _ in range(L)]
        phi = [float(rng.randint(1, 3)) for _ in range(L)]
        beta = [float(rng.randint(0, 6)) for _ in range(M)]
        value, intervals = binding.select_layers(nu, phi, beta, lib)
        assert value == osel.dp_naive(nu, phi, beta)[M][L]
        check_solution(nu, phi, beta, value, intervals)
    # a model-sized instance: 400 layers, 6 verifiers
    L, M = 400, 6
    nu = [rng.random() ** 3 for _ in range(L)]
    phi = [1.0 + rng.random() for _ in range(L)]
    beta = [20.0 + 10 * rng.random() for _ in range(M)]
    value, intervals = binding.select_layers(nu, phi, beta, lib)
    assert value == pytest.approx(osel.dp_naive(nu, phi, beta)[M][L], rel=1e-12)
    check_solution(nu, phi, beta, value, intervals)
    # degenerate inputs
    assert binding.select_layers([], [], [1.0], lib) == (0.0, [None])
    assert binding.select_layers([1.0], [1.0], [], lib)[0] == 0.0
    with pytest.raises(binding.TcError):
        binding.select_layers([1.0], [0.0], [1.0], lib)
    with pytest.raises(binding.TcError):
        binding.select_layers([-1.0], [1.0], [1.0], lib)
