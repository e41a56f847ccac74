"""Pins for the oracle's pairing layer (App. E) and the pairing form of Ver (Def. 4.1), CPU only.

What fixes the map from outside: the field tower's defining relations, the group orders, the properties App. E
lists (bilinearity in both arguments, non-degeneracy, e(S, O) = e(O, T) = 1, inverses, products), and agreement of
the pairing check with the trapdoor form of the same verification equation on honest and tampered openings."""
import random

import numpy as np

import tc_inputs
from oracle import bls12_381 as ec
from oracle import pairing as pr
from oracle import tc
from oracle.bls12_381 import P, R

TAU = tc_inputs.trapdoors()


def test_tower_relations():
    w = [0, 1] + [0] * 10
    w6 = pr.F12_ONE
    for _ in range(6):
        w6 = pr.f12_mul(w6, w)
    u = pr.f12_sub(w6, pr.F12_ONE)                      # u = w^6 - 1
    assert pr.f12_mul(u, u) == pr.f12_from_fp(P - 1)    # u^2 = -1
    assert pr.f12_from_f2((3, 5)) == pr.f12_add(pr.f12_from_fp(3), pr.f12_mul(pr.f12_from_fp(5), u))
    rng = random.Random(1)
    a2, b2 = (rng.randrange(P), rng.randrange(P)), (rng.randrange(P), rng.randrange(P))
    # the embedding Fp2 -> Fp12 is a ring map
    assert pr.f12_from_f2(pr.f2_mul(a2, b2)) == pr.f12_mul(pr.f12_from_f2(a2), pr.f12_from_f2(b2))
    assert pr.f2_mul(a2, pr.f2_inv(a2)) == pr.F2_ONE
    x = [rng.randrange(P) for _ in range(12)]
    y = [rng.randrange(P) for _ in range(12)]
    z = [rng.randrange(P) for _ in range(12)]
    assert pr.f12_mul(x, pr.f12_inv(x)) == pr.F12_ONE
    assert pr.f12_mul(pr.f12_mul(x, y), z) == pr.f12_mul(x, pr.f12_mul(y, z))
    assert pr.f12_mul(x, pr.f12_add(y, z)) == pr.f12_add(pr.f12_mul(x, y), pr.f12_mul(x, z))
    # Fermat in Fp12 on a sparse element (cheap enough): x^(p^12 - 1) = 1 is implied by the group order; here p-th
    # power of an Fp element is itself and the p^2-th power fixes the embedded Fp2
    e2 = pr.f12_from_f2(a2)
    assert pr.f12_pow(e2, P * P) == e2


def test_g2_generator_and_untwist():
    assert pr.g2_is_on_curve(pr.G2)
    assert pr.g2_mul(R - 1, pr.G2) == pr.g2_neg(pr.G2)            # order divides r (prime), and is not 1
    assert pr.g2_add(pr.g2_mul(R - 1, pr.G2), pr.G2) is ec.INF
    q = pr.g2_mul(0xC0FFEE, pr.G2)
    assert pr.g2_is_on_curve(q)
    x, y = pr.untwist(q)                                          # lands on E: y^2 = x^3 + 4 over Fp12
    assert pr.f12_mul(y, y) == pr.f12_add(pr.f12_mul(pr.f12_mul(x, x), x), pr.f12_from_fp(4))
    # the group law commutes with the untwist (it is an isomorphism of curves)
    q2 = pr.g2_mul(77, pr.G2)
    (x1, y1), (x2, y2) = pr.untwist(q), pr.untwist(q2)
    lam = pr.f12_mul(pr.f12_sub(y2, y1), pr.f12_inv(pr.f12_sub(x2, x1)))
    x3 = pr.f12_sub(pr.f12_sub(pr.f12_mul(lam, lam), x1), x2)
    assert x3 == pr.untwist(pr.g2_add(q, q2))[0]
    assert pr.g2_from_bytes(pr.g2_to_bytes(q)) == q and pr.g2_from_bytes(bytes(192)) is ec.INF


def test_pairing_properties():
    e = pr.pairing(ec.G1, pr.G2)
    assert e != pr.F12_ONE                                        # non-degenerate
    assert pr.f12_pow(e, R) == pr.F12_ONE                         # G_T has order r
    a, b = 0x1234567, 0x89ABCDE
    pa, qb = ec.mul(a, ec.G1), pr.g2_mul(b, pr.G2)
    assert pr.pairing(pa, pr.G2) == pr.f12_pow(e, a)              # linear in the first argument
    assert pr.pairing(ec.G1, qb) == pr.f12_pow(e, b)              # and in the second
    assert pr.pairing(pa, qb) == pr.f12_pow(e, a * b % R)
    # e(S, T^-1) = e(S^-1, T) = e(S, T)^-1
    einv = pr.f12_inv(pr.pairing(pa, qb))
    assert pr.pairing(ec.neg(pa), qb) == einv and pr.pairing(pa, pr.g2_neg(qb)) == einv
    # products: prod e(S_i, T) = e(sum S_i, T)
    s1, s2 = ec.mul(11, ec.G1), ec.mul(R - 5, ec.G1)
    assert pr.pairing_product([(s1, qb), (s2, qb)]) == pr.pairing(ec.add(s1, s2), qb)
    # identities on either side give 1
    assert pr.pairing(ec.INF, qb) == pr.F12_ONE and pr.pairing(pa, ec.INF) == pr.F12_ONE


def test_pairing_verification_matches_the_trapdoor_form():
    shape = (3, 4)
    pp = tc.setup(shape, TAU)
    vkey = pr.verifier_key(TAU[:2])
    assert vkey[0] == pr.g2_mul(TAU[0], pr.G2)
    rng = np.random.default_rng(3)
    T = rng.integers(-128, 128, size=shape)
    C = tc.commit(pp, T)
    kappa = (1, 2)
    y, pi = tc.open_(pp, T, kappa)
    assert tc.verify(pp, C, kappa, y, pi)
    assert pr.verify(vkey, C, kappa, y, pi)
    # tampering: value, one proof element, the commitment, the position
    assert not pr.verify(vkey, C, kappa, (y + 1) % R, pi)
    assert not pr.verify(vkey, C, kappa, y, [pi[0], ec.add(pi[1], ec.G1)])
    assert not pr.verify(vkey, ec.add(C, ec.G1), kappa, y, pi)
    assert not pr.verify(vkey, C, (1, 1), y, pi)
    # order 1 (a vector commitment, Def. 2.2) and an opening whose quotient vanishes (constant tensor: pi = O)
    pp1 = tc.setup((5,), TAU)
    v = rng.integers(-9, 9, size=(5,))
    y1, pi1 = tc.open_(pp1, v, (4,))
    assert pr.verify(vkey, tc.commit(pp1, v), (4,), y1, pi1)
    const = np.full(shape, 7)
    yc, pic = tc.open_(pp, const, (0, 0))
    assert all(p is ec.INF for p in pic) and pr.verify(vkey, tc.commit(pp, const), (0, 0), yc, pic)
