"""The library's field / curve headers, compiled for the host with g++, against the oracle.

The HIP kernels inline these same functions; this CPU test finds arithmetic mistakes
(carry handling, exceptional cases of the group law, the G1 -> Fr map) without a GPU."""
import ctypes
import os
import random
import subprocess

import pytest

from oracle import bls12_381 as ec
from oracle import terkle
from oracle.bls12_381 import P, R

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "hostmath", "hostmath.cpp")
LIB = os.path.join(HERE, "hostmath", "libhostmath.so")


@pytest.fixture(scope="module")
def hm():
    hdrs = [os.path.join(HERE, "..", "paper_2602_12630_amd", "csrc", h) for h in ("field.h", "g1.h", "constants.h", "kernels.h", "rt.h", "pairing.h")]
    newest = max(os.path.getmtime(f) for f in [SRC] + hdrs)
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < newest:
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", LIB, SRC])
    return ctypes.CDLL(LIB)


def _b(x, n):
    return (ctypes.c_uint8 * n).from_buffer_copy(int(x).to_bytes(n, "little"))


def _call2(fn, a, b, n):
    out = (ctypes.c_uint8 * n)()
    fn(_b(a, n), _b(b, n), out)
    return int.from_bytes(bytes(out), "little")


def test_fp64_product_columns_stay_exact():
    """The FP64 form of the Fp product sums whole columns of 24-bit limb products in a double: the largest
    column any two operands below the modulus can produce, with the reduction terms and the carry, must stay
    below 2^53."""
    top = P >> 360                                   # the 16th limb of an operand is at most that of the modulus
    limb = (1 << 24) - 1
    p24 = [(P >> (24 * j)) & limb for j in range(16)]
    worst, carry = 0, 0
    for k in range(31):
        lo, hi = max(0, k - 15), min(k, 15)
        ab = sum((top if i == 15 else limb) * (top if k - i == 15 else limb) for i in range(lo, hi + 1))
        mp = sum(limb * p24[k - i] for i in range(lo, hi + 1))
        column = ab + mp + carry
        worst = max(worst, column)
        carry = column >> 24
    assert worst < 1 << 53


def test_fp_fr_arithmetic(hm):
    rng = random.Random(1)
    edge_p = [0, 1, 2, P - 1, P - 2, (P - 1) // 2, (1 << 380), 0xFFFFFFFF, (1 << 352) - 1, (1 << 380) - 1]
    vals = edge_p + [rng.randrange(P) for _ in range(60)]
    for a in vals:
        for b in edge_p + [rng.randrange(P) for _ in range(4)]:
            assert _call2(hm.hm_fp_mul, a, b, 48) == a * b % P                   # 64-bit limbs (host code)
            assert _call2(hm.hm_fp_mul_limbs32, a, b, 48) == a * b % P           # the 32-bit-limb form of the kernels
            assert _call2(hm.hm_fp_mul_f64, a, b, 48) == a * b % P               # 24-bit limbs in doubles (doubling chains)
            assert _call2(hm.hm_fp_sqr_f64, a, b, 48) == a * a % P
            assert _call2(hm.hm_fp_add, a, b, 48) == (a + b) % P
            assert _call2(hm.hm_fp_sub, a, b, 48) == (a - b) % P
    edge_r = [0, 1, 2, R - 1, R - 2, (1 << 254), 0xFFFFFFFF]
    for a in edge_r + [rng.randrange(R) for _ in range(60)]:
        for b in edge_r + [rng.randrange(R) for _ in range(4)]:
            assert _call2(hm.hm_fr_mul, a, b, 32) == a * b % R
            assert _call2(hm.hm_fr_add, a, b, 32) == (a + b) % R
            assert _call2(hm.hm_fr_sub, a, b, 32) == (a - b) % R
    for a in (1, 2, P - 1, rng.randrange(1, P)):
        out = (ctypes.c_uint8 * 48)()
        hm.hm_fp_inv(_b(a, 48), out)
        assert int.from_bytes(bytes(out), "little") * a % P == 1
    for a in (1, 2, 3, P - 1, P - 2, (P - 1) // 2, 1 << 380, rng.randrange(1, P), rng.randrange(1, P)):
        out = (ctypes.c_uint8 * 48)()
        hm.hm_fp_inv_binary(_b(a, 48), out)
        assert int.from_bytes(bytes(out), "little") == pow(a, -1, P)
    for a in (1, 2, R - 1, 1 << 254, rng.randrange(1, R), rng.randrange(1, R)):
        out = (ctypes.c_uint8 * 32)()
        hm.hm_fr_inv_binary(_b(a, 32), out)
        assert int.from_bytes(bytes(out), "little") == pow(a, -1, R)
    for fn_p, fn_r in ((hm.hm_fp_inv_gcd, hm.hm_fr_inv_gcd),):
        edge = [1, 2, 3, (1 << 32), (1 << 62) + 1, (1 << 63) + 5, (1 << 64) - 1, 1 << 64]
        for a in edge + [P - 1, P - 2, (P - 1) // 2, 1 << 380] + [rng.randrange(1, P) for _ in range(300)] + \
                [rng.randrange(1, 1 << rng.randrange(1, 381)) for _ in range(300)]:
            out = (ctypes.c_uint8 * 48)()
            fn_p(_b(a, 48), out)
            assert int.from_bytes(bytes(out), "little") == pow(a, -1, P)
        for a in edge + [R - 1, R - 2, 1 << 254] + [rng.randrange(1, R) for _ in range(300)] + \
                [rng.randrange(1, 1 << rng.randrange(1, 255)) for _ in range(300)]:
            out = (ctypes.c_uint8 * 32)()
            fn_r(_b(a, 32), out)
            assert int.from_bytes(bytes(out), "little") == pow(a, -1, R)
    for v in (0, 1, -1, 127, -128, 32767, -32768, 2**31 - 1, -(2**31)):
        out = (ctypes.c_uint8 * 32)()
        hm.hm_fr_from_i32(ctypes.c_int32(v), out)
        assert int.from_bytes(bytes(out), "little") == v % R


def _pt(fn, *args):
    out = (ctypes.c_uint8 * 96)()
    fn(*args, out)
    return ec.g1_from_bytes(bytes(out))


def _pb(pt):
    return (ctypes.c_uint8 * 96).from_buffer_copy(ec.g1_to_bytes(pt))


def test_group_law_including_exceptional_cases(hm):
    rng = random.Random(2)
    assert _pt(hm.hm_g1_generator) == ec.G1
    pts = [ec.mul(rng.randrange(1, R), ec.G1) for _ in range(5)]
    for mode in (0, 1, 2):
        for a in pts:
            assert _pt(hm.hm_g1_add, _pb(a), _pb(a), mode) == ec.add_affine(a, a)                 # P + P
            assert _pt(hm.hm_g1_add, _pb(a), _pb(ec.neg(a)), mode) is ec.INF                      # P + (-P)
            assert _pt(hm.hm_g1_add, _pb(a), _pb(ec.INF), mode) == a                              # P + O
            assert _pt(hm.hm_g1_add, _pb(ec.INF), _pb(a), mode) == a                              # O + P
            for b in pts:
                assert _pt(hm.hm_g1_add, _pb(a), _pb(b), mode) == ec.add_affine(a, b)
        assert _pt(hm.hm_g1_add, _pb(ec.INF), _pb(ec.INF), mode) is ec.INF
    for k in (0, 1, 2, 3, R - 1, rng.randrange(R), 1 << 200):
        assert _pt(hm.hm_g1_mul, _b(k, 32), _pb(pts[0])) == ec.mul_affine(k, pts[0])

def test_cooperative_reduction(hm):
    """Sums of up to 256 points through the shared-addition kernel, with the operand patterns that leave the
    regular chord rule: identities anywhere, equal neighbours (tangent rule), opposite neighbours, everything
    cancelling."""
    rng = random.Random(5)
    base = [ec.mul(rng.randrange(1, R), ec.G1) for _ in range(6)]

    def run(points, spread):
        buf = b"".join(ec.g1_to_bytes(p) for p in points)
        arr = (ctypes.c_uint8 * max(len(buf), 1)).from_buffer_copy(buf or b"\0")
        out = (ctypes.c_uint8 * 96)()
        hm.hm_coop_reduce(arr, len(points), spread, out)
        return ec.g1_from_bytes(bytes(out))

    def want(points):
        acc = ec.INF
        for p in points:
            acc = ec.add_affine(acc, p)
        return acc

    cases = [
        [],
        [base[0]],
        [base[0], base[1]],
        [base[0], base[0]],                                  # tangent rule at the first level
        [base[0], ec.neg(base[0])],                          # opposite points
        [ec.INF, base[2]],
        [base[2], ec.INF],
        [ec.INF, ec.INF, ec.INF],
        [base[0], base[1], base[0], base[1]],                # equal partial sums one level up
        [base[0], base[1], ec.neg(base[0]), ec.neg(base[1])],
        [base[i % 6] for i in range(17)],
        [base[rng.randrange(6)] if rng.random() < 0.6 else ec.INF for _ in range(255)],
        [ec.mul(i + 1, base[3]) for i in range(64)] + [ec.neg(ec.mul(i + 1, base[3])) for i in range(64)],
        [base[rng.randrange(6)] for _ in range(256)],
    ]
    for spread in (0, 1):
        for pts in cases:
            got = run(pts, spread)
            w = want(pts)
            assert (got is ec.INF and w is ec.INF) or got == w, (len(pts), spread)


def test_pairing_building_blocks(hm):
    """Inside the host pairing: the verifier's short final exponentiation is the cube of the plain one, the
    p-power map equals the power by p, applying it twice equals the p^2-power map, inversion inverts."""
    rng = random.Random(8)
    for _ in range(2):
        pt = ec.mul(rng.randrange(1, R), ec.G1)
        assert hm.hm_final_exponentiation_forms(_pb(pt), rng.randrange(1, 1 << 32)) == 15


def test_phi_map(hm):
    rng = random.Random(3)
    for pt in [ec.INF, ec.G1, ec.neg(ec.G1)] + [ec.mul(rng.randrange(1, R), ec.G1) for _ in range(20)]:
        out = (ctypes.c_uint8 * 32)()
        hm.hm_phi(_pb(pt), out)
        assert int.from_bytes(bytes(out), "little") == terkle.phi(pt)
