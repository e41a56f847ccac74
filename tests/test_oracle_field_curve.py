"""Pins for the oracle's field / curve layer (CPU only).

What fixes the expected values here is outside the oracle: the BLS family
polynomials r(z), p(z), the curve equation, the group order, group axioms, and
agreement of two independently written laws (affine chord-and-tangent in Python
ints, Jacobian in Python ints, Jacobian on 64-bit limbs in C)."""
import random

import pytest

from oracle import bls12_381 as ec
from oracle import cbind


def is_probable_prime(n, rounds=24):
    if n < 2:
        return False
    for q in (2, 3, 5, 7, 11, 13, 17, 19, 23, 29):
        if n % q == 0:
            return n == q
    d, s = n - 1, 0
    while d % 2 == 0:
        d //= 2
        s += 1
    rng = random.Random(7)
    for _ in range(rounds):
        a = rng.randrange(2, n - 1)
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(s - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


def test_constants_from_bls_parameter():
    z = -0xD201000000010000
    r = z**4 - z**2 + 1
    p = (z - 1) ** 2 * r // 3 + z
    assert ((z - 1) ** 2 * r) % 3 == 0
    assert r == ec.R == 0x73EDA753299D7D483339D80809A1D80553BDA402FFFE5BFEFFFFFFFF00000001
    assert p == ec.P
    assert p.bit_length() == 381 and r.bit_length() == 255
    assert is_probable_prime(p) and is_probable_prime(r)
    assert p % 4 == 3
    # curve order: #E(Fp) = p + 1 - t with trace t = z + 1, and it factors as h * r
    assert p + 1 - (z + 1) == ec.COFACTOR * r


def test_generator_on_curve_and_of_order_r():
    assert ec.is_on_curve(ec.G1)
    assert (ec.G1_Y**2 - ec.G1_X**3 - 4) % ec.P == 0
    assert ec.mul_affine(ec.R - 1, ec.G1) == ec.neg(ec.G1)        # so [r]G = O
    assert ec.add_affine(ec.mul_affine(ec.R - 1, ec.G1), ec.G1) is ec.INF
    assert ec.G1_Y <= (ec.P - 1) // 2


def test_affine_and_jacobian_laws_agree():
    rng = random.Random(11)
    pts = [ec.mul_affine(rng.randrange(1, ec.R), ec.G1) for _ in range(6)]
    for a in pts:
        assert ec.is_on_curve(a)
        assert ec.from_jac(ec.jac_double(ec.to_jac(a))) == ec.add_affine(a, a)
        assert ec.add(a, ec.neg(a)) is ec.INF
        assert ec.add(a, ec.INF) == a and ec.add(ec.INF, a) == a
        for b in pts:
            assert ec.add(a, b) == ec.add_affine(a, b)
    # Jacobian inputs with Z != 1 on both sides
    a, b = pts[0], pts[1]
    ja = ec.jac_double(ec.to_jac(a))
    jb = ec.jac_add(ec.to_jac(b), ec.to_jac(a))
    assert ec.from_jac(ec.jac_add(ja, jb)) == ec.add_affine(ec.add_affine(a, a), ec.add_affine(a, b))
    # equal points reached through different Z
    assert ec.from_jac(ec.jac_add(ja, ec.to_jac(ec.add_affine(a, a)))) == ec.mul_affine(4, a)


def test_group_axioms_and_scalar_mult():
    rng = random.Random(12)
    a, b, c = (ec.mul(rng.randrange(1, ec.R), ec.G1) for _ in range(3))
    assert ec.add(ec.add(a, b), c) == ec.add(a, ec.add(b, c))
    assert ec.add(a, b) == ec.add(b, a)
    k1, k2 = rng.randrange(ec.R), rng.randrange(ec.R)
    assert ec.mul(k1 + k2, ec.G1) == ec.add(ec.mul(k1, ec.G1), ec.mul(k2, ec.G1))
    assert ec.mul(k1 * k2, ec.G1) == ec.mul(k1, ec.mul(k2, ec.G1))
    assert ec.mul(k1, ec.G1) == ec.mul_affine(k1, ec.G1)
    assert ec.mul(0, ec.G1) is ec.INF and ec.mul(ec.R, ec.G1) is ec.INF
    assert ec.mul(5, ec.G1) == ec.add(ec.add(ec.add(ec.add(ec.G1, ec.G1), ec.G1), ec.G1), ec.G1)
    assert ec.msm_naive([3, ec.R - 2], [a, b]) == ec.sub(ec.mul(3, a), ec.mul(2, b))


def test_encodings_roundtrip_and_reject():
    a = ec.mul(123456789, ec.G1)
    assert ec.g1_from_bytes(ec.g1_to_bytes(a)) == a
    assert ec.g1_from_bytes(bytes(96)) is ec.INF and ec.g1_to_bytes(ec.INF) == bytes(96)
    bad = bytearray(ec.g1_to_bytes(a))
    bad[0] ^= 1
    with pytest.raises(ValueError):
        ec.g1_from_bytes(bytes(bad))
    assert ec.fr_from_bytes(ec.fr_to_bytes(ec.R - 1)) == ec.R - 1
    with pytest.raises(ValueError):
        ec.fr_from_bytes(ec.R.to_bytes(32, "little"))


def test_c_oracle_field_and_group_match_python_ints():
    rng = random.Random(13)
    edge = [0, 1, 2, ec.P - 1, ec.P - 2, (1 << 380), (1 << 381) - 1 - ec.P]
    for a in edge + [rng.randrange(ec.P) for _ in range(40)]:
        for b in edge[:4] + [rng.randrange(ec.P) for _ in range(3)]:
            assert cbind.fp_mul(a % ec.P, b % ec.P) == (a * b) % ec.P
    edge_r = [0, 1, ec.R - 1, (1 << 254), ec.R - 2]
    for a in edge_r + [rng.randrange(ec.R) for _ in range(40)]:
        for b in edge_r + [rng.randrange(ec.R) for _ in range(3)]:
            assert cbind.fr_mul(a, b) == a * b % ec.R
    for a in (1, 2, ec.P - 1, rng.randrange(1, ec.P)):
        assert cbind.fp_inv(a) * a % ec.P == 1
    assert cbind.g1_generator() == ec.G1
    pts = [ec.mul_affine(rng.randrange(1, ec.R), ec.G1) for _ in range(4)]
    for a in pts:
        assert cbind.g1_add(a, a) == ec.add_affine(a, a)
        assert cbind.g1_add(a, ec.neg(a)) is ec.INF
        assert cbind.g1_add(a, ec.INF) == a and cbind.g1_add(ec.INF, a) == a
        for b in pts:
            assert cbind.g1_add(a, b) == ec.add_affine(a, b)
    for k in (0, 1, 2, ec.R - 1, rng.randrange(ec.R)):
        assert cbind.g1_mul(k, pts[0]) == ec.mul_affine(k, pts[0])
