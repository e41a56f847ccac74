"""Pins for the oracle's tensor commitment (Def. 4.1), CPU only.

Expected values come from outside the functions under test: brute-force
interpolation by Gaussian elimination on the full Vandermonde system, the
m = 1 reduction to the vector commitment of Def. 2.2 worked out with explicit
polynomial long division, linearity in the exponent, special tensors with a
closed-form commitment, the correctness and binding statements, the
post-condition of Algorithm 1, and agreement of independently written routes."""
import itertools
import random

import numpy as np
import pytest

import tc_inputs
from oracle import bls12_381 as ec
from oracle import cbind, tc
from oracle.bls12_381 import R

TAU = tc_inputs.trapdoors()


def solve_mod_r(A, b):
    """Gaussian elimination over Fr (test-side, independent of the oracle)."""
    n = len(A)
    M = [[x % R for x in row] + [bi % R] for row, bi in zip(A, b)]
    for c in range(n):
        piv = next(i for i in range(c, n) if M[i][c])
        M[c], M[piv] = M[piv], M[c]
        inv = pow(M[c][c], -1, R)
        M[c] = [x * inv % R for x in M[c]]
        for i in range(n):
            if i != c and M[i][c]:
                f = M[i][c]
                M[i] = [(x - f * y) % R for x, y in zip(M[i], M[c])]
    return [row[n] for row in M]


def brute_force_coeffs(T, shape):
    """Solve sum_k a_k prod_j zeta^(k_j) = T[i] over all grid points at once."""
    idx = list(itertools.product(*[range(d) for d in shape]))
    A = []
    for i in idx:
        row = []
        for k in idx:
            v = 1
            for ij, kj in zip(i, k):
                v = v * pow(ij + 1, kj, R) % R
            row.append(v)
        A.append(row)
    return solve_mod_r(A, [int(v) for v in np.asarray(T).reshape(-1)])


def eval_brute(coeffs, shape, x):
    total = 0
    for k, c in zip(itertools.product(*[range(d) for d in shape]), coeffs):
        term = c
        for xj, kj in zip(x, k):
            term = term * pow(xj, kj, R) % R
        total = (total + term) % R
    return total


SHAPES = [(2, 2), (2, 3), (2, 2, 2), (3, 4), (5,), (2, 1, 3), (2, 2, 2, 2)]


@pytest.mark.parametrize("shape", SHAPES)
def test_brute_force_interpolation_and_commitment(shape):
    T = tc_inputs.int16_uniform(shape, 100 + len(shape))
    pp = tc.setup(shape, TAU)
    a = brute_force_coeffs(T, shape)
    assert tc.interpolate(T, shape) == a
    # f_T reproduces T on the grid (negatives as r - |x|)
    for i in itertools.product(*[range(d) for d in shape]):
        assert eval_brute(a, shape, [ij + 1 for ij in i]) == int(T[i]) % R
    # C_T = [f_T(tau)]G, with f_T(tau) from the brute-force coefficients
    s = eval_brute(a, shape, TAU[: len(shape)])
    assert tc.f_at_tau(pp, T) == s
    expect = ec.mul_affine(s, ec.G1)
    assert tc.commit(pp, T) == expect
    assert tc.commit_literal(pp, T) == expect
    assert tc.commit_lagrange_naive(pp, T) == expect
    assert cbind.commit(pp, T, 2) == expect


@pytest.mark.parametrize("shape", SHAPES + [(9,), (1,), (4, 1, 3)])
@pytest.mark.parametrize("form", sorted(tc.INTERPOLATION_FORMS))
def test_interpolation_forms_of_app_c(shape, form):
    """Newton, Gregory and barycentric interpolation (App. C) are three ways to the same polynomial: each
    must return the coefficients of the brute-force Vandermonde solve, and a textbook special case each."""
    T = tc_inputs.int16_uniform(shape, 300 + len(shape))
    assert tc.interpolate_form(T, shape, form) == brute_force_coeffs(T, shape)
    line = tc.INTERPOLATION_FORMS[form]
    # samples of X^2 on the nodes 1, 2, 3, 4: coefficients (0, 0, 1, 0); a constant line: (c, 0, 0)
    assert line([1, 4, 9, 16]) == [0, 0, 1, 0]
    assert line([7, 7, 7]) == [7, 0, 0]
    # the line through (1, 3) and (2, 5) is 1 + 2 X
    assert line([3, 5]) == [1, 2]


def test_monomial_srs_is_the_setup_of_def_4_1():
    pp = tc.setup((2, 3), TAU)
    M = pp.srs_monomial()
    for i1 in range(2):
        for i2 in range(3):
            assert M[i1 * 3 + i2] == ec.mul_affine(pow(TAU[0], i1, R) * pow(TAU[1], i2, R) % R, ec.G1)


def test_lagrange_basis_forms_agree():
    for d in (1, 2, 3, 7, 16):
        assert tc.bary_weights(d) == tc.bary_weights_direct(d)
        x = TAU[1]
        ell = tc.lagrange_at(d, x)
        assert ell == tc.lagrange_at_direct(d, x)
        assert sum(ell) % R == 1                                     # partition of unity
        # reproduces polynomials of degree < d: sum_i zeta_i^e l_i(x) = x^e
        for e in range(d):
            assert sum(pow(i + 1, e, R) * ell[i] for i in range(d)) % R == pow(x, e, R)
    with pytest.raises(ValueError):
        tc.lagrange_at(4, 3)                                         # on the grid
    with pytest.raises(ValueError):
        tc.setup((4,), [2])


def poly_divmod_linear(coeffs, w):
    """Textbook synthetic division of a univariate polynomial (low degree first) by (X - w)."""
    q = [0] * (len(coeffs) - 1)
    carry = 0
    for e in range(len(coeffs) - 1, 0, -1):
        carry = (coeffs[e] + carry * w) % R
        q[e - 1] = carry
    rem = (coeffs[0] + carry * w) % R
    return q, rem


def test_m1_reduces_to_kzg_vector_commitment():
    """Def. 2.2: c = g^{f(tau)}, pi_i = g^{h_i(tau)}, h_i = (f - y)/(X - omega_i);
    check e(C g^{-y}, g) = e(pi, g^{tau - omega}) in exponent form."""
    d = 6
    v = tc_inputs.int8_uniform((d,), 42)
    pp = tc.setup((d,), TAU)
    coeffs = brute_force_coeffs(v, (d,))
    tau = TAU[0]
    f_tau = sum(c * pow(tau, e, R) for e, c in enumerate(coeffs)) % R
    C = tc.commit(pp, v)
    assert C == ec.mul_affine(f_tau, ec.G1)
    for i in range(d):
        omega = i + 1
        q, rem = poly_divmod_linear(coeffs, omega)
        assert rem == int(v[i]) % R
        h_tau = sum(c * pow(tau, e, R) for e, c in enumerate(q)) % R
        y, proof = tc.open_(pp, v, (i,))
        assert y == rem and proof == [ec.mul_affine(h_tau, ec.G1)]
        assert (f_tau - y) % R == h_tau * (tau - omega) % R
        assert tc.verify(pp, C, (i,), y, proof)
        assert tc.open_literal(pp, v, (i,)) == (y, proof)


def test_linearity_in_the_exponent():
    shape = (3, 4, 2)
    pp = tc.setup(shape, TAU)
    T = tc_inputs.int16_uniform(shape, 1).astype(np.int64)
    U = tc_inputs.int16_uniform(shape, 2).astype(np.int64)
    a, b = 37, -91
    lhs = tc.commit(pp, (a * T + b * U))
    rhs = ec.add(ec.mul(a % R, tc.commit(pp, T)), ec.mul(b % R, tc.commit(pp, U)))
    assert lhs == rhs
    assert tc.commit_lagrange_naive(pp, a * T + b * U) == rhs


@pytest.mark.parametrize("shape", [(4,), (3, 5), (4, 16, 16), (2, 3, 2, 2)])
def test_special_tensors(shape):
    pp = tc.setup(shape, TAU)
    n = tc.prod(shape)
    assert tc.commit(pp, np.zeros(shape, np.int16)) is ec.INF
    for c in (1, -1, 77, -128):
        assert tc.commit(pp, np.full(shape, c, np.int16)) == ec.mul_affine(c % R, ec.G1)   # constant => [c]G
    if n <= 64:
        S = pp.srs_lagrange(0)
        acc = ec.INF
        for s in S:
            acc = ec.add_affine(acc, s)
        assert acc == ec.G1                                          # sum_i S[i] = G
        for f in (0, n // 2, n - 1):
            onehot = np.zeros(n, np.int16)
            onehot[f] = 1
            assert tc.commit(pp, onehot.reshape(shape)) == S[f]
            assert S[f] == ec.mul_affine(pp.lagrange_scalar(tc.multi_index(f, shape)), ec.G1)
        # suffix tables are partial sums of the full table (partition of unity on the dropped axes)
        if len(shape) > 1:
            inner = tc.prod(shape[1:])
            S1 = pp.srs_lagrange(1)
            for t in range(inner):
                acc = ec.INF
                for k in range(shape[0]):
                    acc = ec.add_affine(acc, S[k * inner + t])
                assert acc == S1[t]


def test_algorithm_1_postcondition_and_layout():
    shape = (3, 4, 2)
    rng = random.Random(5)
    a = [rng.randrange(R) for _ in range(tc.prod(shape))]
    # layout: index(i) = sum_j i_j * prod_{t>j} d_t, last exponent fastest
    assert tc.flat_index((1, 2, 1), shape) == 1 * 8 + 2 * 2 + 1
    assert tc.multi_index(13, shape) == (1, 2, 1)
    for axis in range(3):
        v = rng.randrange(R)
        q, r = tc.divide_by_linear(a, shape, axis, v)
        # r is free of x_axis
        for f, c in enumerate(r):
            if tc.multi_index(f, shape)[axis] != 0:
                assert c == 0
        # q has degree <= d-2 in x_axis
        for f, c in enumerate(q):
            if tc.multi_index(f, shape)[axis] == shape[axis] - 1:
                assert c == 0
        for _ in range(3):
            x = [rng.randrange(R) for _ in shape]
            lhs = eval_brute(a, shape, x)
            rhs = (eval_brute(q, shape, x) * (x[axis] - v) + eval_brute(r, shape, x)) % R
            assert lhs == rhs
        # remainder = f with x_axis := v
        x = [rng.randrange(R) for _ in shape]
        xv = list(x)
        xv[axis] = v
        assert eval_brute(r, shape, x) == eval_brute(a, shape, xv)


@pytest.mark.parametrize("shape", [(3, 4), (2, 3, 2), (4, 4), (2, 2, 2, 2)])
def test_open_routes_agree_and_verify(shape):
    pp = tc.setup(shape, TAU)
    T = tc_inputs.int16_uniform(shape, 9)
    C = tc.commit(pp, T)
    coeffs = brute_force_coeffs(T, shape)
    for kappa in tc_inputs.opening_positions(shape, 3, 5) + [tuple(0 for _ in shape), tuple(d - 1 for d in shape)]:
        y, proof = tc.open_(pp, T, kappa)
        assert y == int(T[kappa]) % R
        assert (y, proof) == tc.open_literal(pp, T, kappa)
        assert (y, proof) == tc.open_eval_form(pp, T, kappa)
        assert len(proof) == len(shape)
        assert tc.verify(pp, C, kappa, y, proof)
        # the identity behind the check, in the exponent: f(tau) - y = sum_i q_i(tau)(tau_i - omega_i)
        _, qs = tc.quotient_scalars(pp, T, kappa)
        s = sum(q * (t - (k + 1)) for q, t, k in zip(qs, pp.tau, kappa)) % R
        assert (eval_brute(coeffs, shape, pp.tau) - y) % R == s
        # quotient values on the grid are values of the Algorithm-1 quotient polynomial
        rem = coeffs
        for i in range(len(shape)):
            q, rem = tc.divide_by_linear(rem, shape, i, kappa[i] + 1)
            qv = tc.quotient_values_on_grid(pp, T, kappa, i)
            sub = shape[i:]
            for f in range(tc.prod(sub)):
                k = tc.multi_index(f, sub)
                pt = [kj + 1 for kj in kappa[:i]] + [kj + 1 for kj in k]
                assert eval_brute(q, shape, pt) == qv[f]


def test_tampering_is_rejected():
    shape = (3, 4)
    pp = tc.setup(shape, TAU)
    T = tc_inputs.int16_uniform(shape, 21)
    C = tc.commit(pp, T)
    kappa = (1, 2)
    y, proof = tc.open_(pp, T, kappa)
    assert tc.verify(pp, C, kappa, y, proof)
    assert not tc.verify(pp, C, kappa, (y + 1) % R, proof)                      # wrong value
    assert not tc.verify(pp, C, (1, 3), y, proof)                               # wrong position
    for i in range(2):
        bad = list(proof)
        bad[i] = ec.add(bad[i], ec.G1)
        assert not tc.verify(pp, C, kappa, y, bad)                              # wrong proof element
    assert not tc.verify(pp, C, kappa, y, proof[:1])
    T2 = T.copy()
    T2[1, 2] += 1                                                               # flipped entry
    C2 = tc.commit(pp, T2)
    assert C2 != C
    assert not tc.verify(pp, C2, kappa, y, proof)
    y2, proof2 = tc.open_(pp, T2, kappa)
    assert not tc.verify(pp, C, kappa, y2, proof2)
    T3 = T.copy()
    T3[0, 0] += 1                                                               # flip elsewhere
    assert not tc.verify(pp, tc.commit(pp, T3), kappa, y, proof)


def test_printed_product_form_does_not_hold_for_m2():
    """Documents the reading taken for Ver: with m = 2 no single quotient satisfies
    f - y = q prod_j (X_j - omega_j): f - y does not vanish on the line X_1 = omega_1."""
    shape = (3, 4)
    T = tc_inputs.int16_uniform(shape, 21)
    coeffs = brute_force_coeffs(T, shape)
    y = int(T[1, 2]) % R
    assert (eval_brute(coeffs, shape, [2, 1]) - y) % R != 0     # X_1 = omega_1 = 2, X_2 = 1 != omega_2


def test_c_oracle_naive_msm_and_closed_form_agree_with_python():
    shape = (4, 16, 16)
    pp = tc.setup(shape, TAU)
    T = tc_inputs.c1_tensor()
    # SRS by the C scalar multiplication, spot-checked against Python ints
    flat = list(range(0, 1024, 97))
    pts = {f: cbind.g1_mul(pp.lagrange_scalar(tc.multi_index(f, shape)), ec.G1) for f in range(1024)}
    for f in flat:
        assert pts[f] == ec.mul(pp.lagrange_scalar(tc.multi_index(f, shape)), ec.G1)
    blob = b"".join(ec.g1_to_bytes(pts[f]) for f in range(1024))
    C_naive, used = cbind.msm_naive(T, blob, 4)
    assert used == 4
    assert C_naive == tc.commit(pp, T) == cbind.commit(pp, T, 3)
    # full-width scalars through the Fr path of the C MSM
    rng = random.Random(3)
    sc = [rng.randrange(R) for _ in range(16)]
    C_fr, _ = cbind.msm_naive(b"".join(ec.fr_to_bytes(s) for s in sc), blob[: 16 * 96], 2)
    assert C_fr == ec.msm_naive(sc, [pts[f] for f in range(16)])
    # int16 tensor at a size with ragged thread split
    X = tc_inputs.int16_uniform((7, 33), 8)
    pp2 = tc.setup((7, 33), TAU)
    assert cbind.f_at_tau(X, (7, 33), pp2.ell, 5) == tc.f_at_tau(pp2, X)
    # openings with the sums in C equal the Python route (and with it Algorithm 1, pinned above), int8 and int16,
    # at corner and interior positions of tensors of order 1 to 3
    for shp, data, kappas in (((7, 33), X, [(0, 0), (6, 32), (3, 17)]), (shape, T, [(3, 15, 15), (1, 0, 7)]),
                              ((12,), tc_inputs.int16_uniform((12,), 9), [(0,), (11,)])):
        ppx = tc.setup(shp, TAU)
        for kappa in kappas:
            assert cbind.open_(ppx, data, kappa, 3) == tc.open_(ppx, data, kappa)
