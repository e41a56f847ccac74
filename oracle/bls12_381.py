"""BLS12-381 field and G1 group layer of the oracle (test infrastructure only).

App. E of the paper fixes the setting (prime-order pairing-friendly groups, the
chord-and-tangent group law) and names BLS12-381 as the curve in use.  In the
usual BLS12-381 naming the group order is `r` and the base-field prime is `p`;
the paper's "prime order p" (Sec. 2, notation) is `r` here.

Everything is Python `int` arithmetic.  Nothing here is tuned; the affine law
is the definition, the Jacobian law is the textbook projective form of it and
is cross-checked against the affine one in the tests.
"""

# --- constants, derived from the BLS parameter z (checked in tests: primality,
# --- on-curve, order) --------------------------------------------------------
Z_BLS = -0xD201000000010000
R = Z_BLS**4 - Z_BLS**2 + 1                       # scalar-field modulus (255 bit)
P = (Z_BLS - 1) ** 2 * R // 3 + Z_BLS             # base-field modulus (381 bit)
B_COEFF = 4                                       # E: y^2 = x^3 + 4
COFACTOR = (Z_BLS - 1) ** 2 // 3
G1_X = 0x17F1D3A73197D7942695638C4FA9AC0FC3688C4F9774B905A14E3A3F171BAC586C55E83FF97A1AEFFB3AF00ADB22C6BB
G1_Y = 0x08B3F481E3AAA0F1A09E30ED741D8AE4FCF5E095D5D00AF600DB18CB2C04B3EDD03CC744A2888AE40CAA232946C5E7E1
G1 = (G1_X, G1_Y)
INF = None                                        # the identity (point at infinity)

FR_BYTES = 32
FP_BYTES = 48
G1_BYTES = 96


# --- scalar field ------------------------------------------------------------
def fr(x):
    return x % R


def fr_inv(x):
    x %= R
    if x == 0:
        raise ZeroDivisionError("inverse of 0 in Fr")
    return pow(x, R - 2, R)                        # Fermat


def fp_inv(x):
    x %= P
    if x == 0:
        raise ZeroDivisionError("inverse of 0 in Fp")
    return pow(x, P - 2, P)


# --- affine chord-and-tangent law (the definition; App. E) --------------------
def is_on_curve(pt):
    if pt is INF:
        return True
    x, y = pt
    return 0 <= x < P and 0 <= y < P and (y * y - x * x * x - B_COEFF) % P == 0


def neg(pt):
    if pt is INF:
        return INF
    x, y = pt
    return (x, (-y) % P)


def add_affine(a, b):
    """a + b by the chord (a != +-b) or the tangent (a == b)."""
    if a is INF:
        return b
    if b is INF:
        return a
    x1, y1 = a
    x2, y2 = b
    if x1 == x2:
        if (y1 + y2) % P == 0:
            return INF                             # b == -a (covers y == 0)
        lam = 3 * x1 * x1 * fp_inv(2 * y1) % P     # tangent slope
    else:
        lam = (y2 - y1) * fp_inv(x2 - x1) % P      # chord slope
    x3 = (lam * lam - x1 - x2) % P
    y3 = (lam * (x1 - x3) - y1) % P
    return (x3, y3)


def mul_affine(k, pt):
    """[k]pt by MSB-first double-and-add with the affine law (slow; small uses)."""
    k %= R
    acc = INF
    for bit in bin(k)[2:] if k else "":
        acc = add_affine(acc, acc)
        if bit == "1":
            acc = add_affine(acc, pt)
    return acc


# --- Jacobian coordinates (X:Y:Z), x = X/Z^2, y = Y/Z^3; Z == 0 is the identity --
J_INF = (1, 1, 0)


def to_jac(pt):
    return J_INF if pt is INF else (pt[0], pt[1], 1)


def from_jac(j):
    X, Y, Z = j
    if Z % P == 0:
        return INF
    zi = fp_inv(Z)
    zi2 = zi * zi % P
    return (X * zi2 % P, Y * zi2 * zi % P)


def jac_double(a):
    X, Y, Z = a
    if Z == 0 or Y == 0:
        return J_INF
    A = X * X % P
    Bq = Y * Y % P
    C = Bq * Bq % P
    D = 2 * ((X + Bq) * (X + Bq) - A - C) % P
    E = 3 * A % P
    X3 = (E * E - 2 * D) % P
    Y3 = (E * (D - X3) - 8 * C) % P
    Z3 = 2 * Y * Z % P
    return (X3, Y3, Z3)


def jac_add(a, b):
    X1, Y1, Z1 = a
    X2, Y2, Z2 = b
    if Z1 == 0:
        return b
    if Z2 == 0:
        return a
    Z1Z1 = Z1 * Z1 % P
    Z2Z2 = Z2 * Z2 % P
    U1 = X1 * Z2Z2 % P
    U2 = X2 * Z1Z1 % P
    S1 = Y1 * Z2 * Z2Z2 % P
    S2 = Y2 * Z1 * Z1Z1 % P
    H = (U2 - U1) % P
    Rr = (S2 - S1) % P
    if H == 0:
        return jac_double(a) if Rr == 0 else J_INF
    HH = H * H % P
    HHH = H * HH % P
    V = U1 * HH % P
    X3 = (Rr * Rr - HHH - 2 * V) % P
    Y3 = (Rr * (V - X3) - S1 * HHH) % P
    Z3 = H * Z1 * Z2 % P
    return (X3, Y3, Z3)


def mul(k, pt):
    """[k]pt, k reduced mod r, MSB-first double-and-add; one inversion at the end."""
    k %= R
    if pt is INF or k == 0:
        return INF
    base = to_jac(pt)
    acc = J_INF
    for bit in bin(k)[2:]:
        acc = jac_double(acc)
        if bit == "1":
            acc = jac_add(acc, base)
    return from_jac(acc)


def add(a, b):
    return from_jac(jac_add(to_jac(a), to_jac(b)))


def sub(a, b):
    return add(a, neg(b))


def msm_naive(scalars, points):
    """sum_i [s_i]P_i, every term by its own double-and-add (Def. 2.2 / Def. 4.1
    'multi-exponentiation', written out term by term)."""
    acc = J_INF
    for s, pt in zip(scalars, points):
        acc = jac_add(acc, to_jac(mul(s, pt)))
    return from_jac(acc)


# --- canonical byte encodings -------------------------------------------------
def fr_to_bytes(x):
    assert 0 <= x < R
    return int(x).to_bytes(FR_BYTES, "little")


def fr_from_bytes(b):
    x = int.from_bytes(bytes(b), "little")
    if len(b) != FR_BYTES or x >= R:
        raise ValueError("non-canonical Fr encoding")
    return x


def g1_to_bytes(pt):
    """x || y, 48 bytes little-endian each; the identity is 96 zero bytes
    ((0,0) is not on y^2 = x^3 + 4, so the encoding is unambiguous)."""
    if pt is INF:
        return bytes(G1_BYTES)
    x, y = pt
    return int(x).to_bytes(FP_BYTES, "little") + int(y).to_bytes(FP_BYTES, "little")


def g1_from_bytes(b):
    b = bytes(b)
    if len(b) != G1_BYTES:
        raise ValueError("G1 encoding must be 96 bytes")
    if b == bytes(G1_BYTES):
        return INF
    x = int.from_bytes(b[:FP_BYTES], "little")
    y = int.from_bytes(b[FP_BYTES:], "little")
    pt = (x, y)
    if not is_on_curve(pt):
        raise ValueError("not a point of E(Fp)")
    return pt
