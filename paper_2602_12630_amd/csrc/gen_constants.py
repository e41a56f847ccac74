"""Generates constants.h for the HIP library (Montgomery constants of BLS12-381).

Run:  python paper_2602_12630_amd/csrc/gen_constants.py
Everything is derived from the BLS parameter z and the G1 generator; nothing is
imported from the test oracle."""
import os

Z = -0xD201000000010000
R_MOD = Z**4 - Z**2 + 1
P_MOD = (Z - 1) ** 2 * R_MOD // 3 + Z
GX = 0x17F1D3A73197D7942695638C4FA9AC0FC3688C4F9774B905A14E3A3F171BAC586C55E83FF97A1AEFFB3AF00ADB22C6BB
GY = 0x08B3F481E3AAA0F1A09E30ED741D8AE4FCF5E095D5D00AF600DB18CB2C04B3EDD03CC744A2888AE40CAA232946C5E7E1


def ec_add(a, b):
    """affine chord-and-tangent on y^2 = x^3 + 4 (only used to pick the endomorphism constant)"""
    if a is None:
        return b
    if b is None:
        return a
    (x1, y1), (x2, y2) = a, b
    if x1 == x2:
        if (y1 + y2) % P_MOD == 0:
            return None
        lam = 3 * x1 * x1 * pow(2 * y1, -1, P_MOD) % P_MOD
    else:
        lam = (y2 - y1) * pow(x2 - x1, -1, P_MOD) % P_MOD
    x3 = (lam * lam - x1 - x2) % P_MOD
    return (x3, (lam * (x1 - x3) - y1) % P_MOD)


def ec_mul(k, pt):
    acc = None
    for bit in bin(k)[2:]:
        acc = ec_add(acc, acc)
        if bit == "1":
            acc = ec_add(acc, pt)
    return acc


def endomorphism():
    """lambda = z^2 - 1 is a primitive cube root of unity mod r; (x, y) -> (beta x, y) is multiplication
    by lambda on G1 for the matching primitive cube root of unity beta mod p."""
    lam = Z * Z - 1
    assert (lam * lam + lam + 1) % R_MOD == 0 and 0 < lam < (1 << 128)
    target = ec_mul(lam, (GX, GY))
    g = 2
    while pow(g, (P_MOD - 1) // 3, P_MOD) == 1:
        g += 1
    beta = pow(g, (P_MOD - 1) // 3, P_MOD)
    for cand in (beta, beta * beta % P_MOD):
        if (cand * GX % P_MOD, GY) == target:
            return lam, cand
    raise AssertionError("no matching cube root of unity")


# G2 generator on the twist y^2 = x^3 + 4 (u + 1) over Fp2 = Fp[u]/(u^2 + 1) (x = x0 + x1 u, y = y0 + y1 u)
G2X = (0x024AA2B2F08F0A91260805272DC51051C6E47AD4FA403B02B4510B647AE3D1770BAC0326A805BBEFD48056C8C121BDB8,
       0x13E02B6052719F607DACD3A088274F65596BD0D09920B61AB5DA61BBDC7F5049334CF11213945D57E5AC7D055D042B7E)
G2Y = (0x0CE5D527727D6E118CC9CDC6DA2E351AADFD9BAA8CBDD3A76D429A695160D12C923AC9CC3BACA289E193548608B82801,
       0x0606C4A02EA734CC32ACD2B02BC28B99CB3E287E85A763AF267492AB572E99AB3F370D275CEC1DA1AAA9075FF05F79BE)


def f2mul(a, b):
    return ((a[0] * b[0] - a[1] * b[1]) % P_MOD, (a[0] * b[1] + a[1] * b[0]) % P_MOD)


def f2pow(a, e):
    out = (1, 0)
    for bit in bin(e)[2:]:
        out = f2mul(out, out)
        if bit == "1":
            out = f2mul(out, a)
    return out


def pairing_constants():
    """gamma = (u + 1)^((p^2 - 1) / 6): with Fp12 = Fp2[w]/(w^6 - (u + 1)) the p^2-power map multiplies the
    coefficient of w^k by gamma^k; the hard part of the final exponentiation is (p^4 - p^2 + 1) / r."""
    xi = (1, 1)
    x3 = f2mul(f2mul(G2X, G2X), G2X)
    assert f2mul(G2Y, G2Y) == ((x3[0] + 4) % P_MOD, (x3[1] + 4) % P_MOD), "G2 generator is not on the twist"
    assert (P_MOD * P_MOD - 1) % 6 == 0
    assert (P_MOD - 1) % 6 == 0
    gamma1 = f2pow(xi, (P_MOD - 1) // 6)
    gamma = f2pow(xi, (P_MOD * P_MOD - 1) // 6)
    assert f2pow(gamma, 6) == (1, 0) and f2pow(gamma, 3) != (1, 0) and f2pow(gamma, 2) != (1, 0)
    assert (P_MOD**4 - P_MOD**2 + 1) % R_MOD == 0
    hard = (P_MOD**4 - P_MOD**2 + 1) // R_MOD
    # three times the hard part splits over the curve parameter (checked here, used by the verifier)
    assert 3 * hard == (Z - 1) ** 2 * (Z + P_MOD) * (Z * Z + P_MOD * P_MOD - 1) + 3
    return gamma1, gamma, hard


def limbs(x, n):
    return ", ".join("0x%08xu" % ((x >> (32 * i)) & 0xFFFFFFFF) for i in range(n))


def block(name, mod, n):
    Rm = 1 << (32 * n)
    inv = (-pow(mod, -1, 1 << 32)) % (1 << 32)
    out = []
    out.append("struct %s {" % name)
    out.append("    static constexpr int N = %d;" % n)
    out.append("    static constexpr uint32_t INV = 0x%08xu;            /* -mod^-1 mod 2^32 */" % inv)
    out.append("    static constexpr uint32_t MOD[%d] = {%s};" % (n, limbs(mod, n)))
    out.append("    static constexpr uint32_t ONE[%d] = {%s};   /* R mod q */" % (n, limbs(Rm % mod, n)))
    out.append("    static constexpr uint32_t R2[%d] = {%s};    /* R^2 mod q */" % (n, limbs(Rm * Rm % mod, n)))
    out.append("    static constexpr uint32_t R3[%d] = {%s};    /* R^3 mod q */" % (n, limbs(pow(Rm, 3, mod), n)))
    out.append("    static constexpr uint32_t MOD_M2[%d] = {%s}; /* q - 2 */" % (n, limbs(mod - 2, n)))
    rounds = -(-(2 * mod.bit_length() - 1) // 30) + 1
    out.append("    static constexpr int GCD_ROUNDS = %d;              /* ceil((2 len(q) - 1) / 30) + 1 */" % rounds)
    out.append("    static constexpr uint32_t GCD_FIX[%d] = {%s}; /* 4^GCD_ROUNDS * R^3 mod q */"
               % (n, limbs(pow(4, rounds, mod) * pow(Rm, 3, mod) % mod, n)))
    out.append("    static constexpr uint32_t HALF[%d] = {%s};  /* (q - 1) / 2 */" % (n, limbs((mod - 1) // 2, n)))
    out.append("};")
    return "\n".join(out)


def limbs28(x, n=14):
    return ", ".join("0x%07x" % ((x >> (28 * i)) & 0xFFFFFFF) for i in range(n))


def block28():
    """Fp in 14 limbs of 28 bits, Montgomery radix 2^392 (the accumulation kernel's second form of the field)."""
    Rm = 1 << 392
    out = []
    out.append("struct Fp28Params {")
    out.append("    static constexpr int N = 14;")
    out.append("    static constexpr int32_t NINV = 0x%07x;              /* -p^-1 mod 2^28 */" % ((-pow(P_MOD, -1, 1 << 28)) % (1 << 28)))
    out.append("    static constexpr int32_t PINV = 0x%07x;              /* p^-1 mod 2^28 */" % pow(P_MOD, -1, 1 << 28))
    out.append("    static constexpr int32_t MOD[14] = {%s};" % limbs28(P_MOD))
    out.append("    static constexpr int32_t ONE[14] = {%s};   /* 2^392 mod p */" % limbs28(Rm % P_MOD))
    rounds = -(-(2 * P_MOD.bit_length() - 1) // 28) + 1
    out.append("    static constexpr int GCD_ROUNDS = %d;                /* ceil((2 len(p) - 1) / 28) + 1 rounds of 28 steps */" % rounds)
    out.append("    static constexpr int32_t INV_FIX[14] = {%s};  /* 2^1168 mod p: 1 / a (mod p) -> the 28-bit form of R^2 / a, R = 2^384 */"
               % limbs28(pow(2, 1168, P_MOD)))
    out.append("};")
    return "\n".join(out)


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    Rp = 1 << 384
    LAM, BETA = endomorphism()
    GAMMA1, GAMMA, HARD = pairing_constants()
    text = [
        "/* GENERATED by gen_constants.py -- do not edit.  BLS12-381 Montgomery constants,",
        " * 32-bit limbs, little-endian limb order.  Fp: R = 2^384; Fr: R = 2^256. */",
        "#pragma once",
        "#include <stdint.h>",
        "namespace tc {",
        block("FpParams", P_MOD, 12),
        block("FrParams", R_MOD, 8),
        block28(),
        "/* G1 generator, Montgomery form */",
        "static constexpr uint32_t G1_GEN_X[12] = {%s};" % limbs(GX * Rp % P_MOD, 12),
        "static constexpr uint32_t G1_GEN_Y[12] = {%s};" % limbs(GY * Rp % P_MOD, 12),
        "/* endomorphism (x, y) -> (beta x, y) = [lambda](x, y), lambda = z^2 - 1 < 2^128 */",
        "static constexpr uint32_t GLV_LAMBDA[4] = {%s};" % limbs(LAM, 4),
        "static constexpr uint32_t GLV_BETA[12] = {%s};      /* Montgomery form */" % limbs(BETA * Rp % P_MOD, 12),
        "/* pairing (host side): G2 generator on the twist, Montgomery form, (c0, c1) of x then of y */",
        "static constexpr uint32_t G2_GEN[4][12] = {%s};"
        % ", ".join("{%s}" % limbs(v * Rp % P_MOD, 12) for v in (G2X[0], G2X[1], G2Y[0], G2Y[1])),
        "/* (u + 1)^((p - 1) / 6), Montgomery form (c0, c1) */",
        "static constexpr uint32_t FROB1_GAMMA[2][12] = {%s};" % ", ".join("{%s}" % limbs(v * Rp % P_MOD, 12) for v in GAMMA1),
        "/* (u + 1)^((p^2 - 1) / 6), Montgomery form (c0, c1) */",
        "static constexpr uint32_t FROB2_GAMMA[2][12] = {%s};" % ", ".join("{%s}" % limbs(v * Rp % P_MOD, 12) for v in GAMMA),
        "/* |z|, the loop length of the Miller function */",
        "static constexpr uint64_t BLS_Z_ABS = 0x%xull;" % abs(Z),
        "/* (p^4 - p^2 + 1) / r, %d bits */" % HARD.bit_length(),
        "static constexpr int HARD_EXP_LIMBS = %d;" % ((HARD.bit_length() + 31) // 32),
        "static constexpr uint32_t HARD_EXP[%d] = {%s};" % ((HARD.bit_length() + 31) // 32, limbs(HARD, (HARD.bit_length() + 31) // 32)),
        "}  // namespace tc",
        "",
    ]
    with open(os.path.join(here, "constants.h"), "w") as f:
        f.write("\n".join(text))


if __name__ == "__main__":
    main()
