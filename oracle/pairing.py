"""Pairing layer of the oracle (test infrastructure only): G2, the target group and the
bilinear map of App. E (pairing-friendly curves), and the pairing form of Ver (Def. 4.1) in
the sum-form reading used throughout this repository:

    e(C - [y]G, H) = prod_i e(pi_i, [tau_i]H - [zeta_i]H)

The paper writes a symmetric pairing e: G x G -> G_T; BLS12-381, which it names, is asymmetric,
so the second arguments live in G2 (generator H) and the public parameters carry [tau_i]H.

Everything is written from the definitions, slowly and plainly:
  * Fp2 = Fp[u]/(u^2 + 1); the sextic twist E': y^2 = x^3 + 4(u + 1) over Fp2 holds G2;
  * Fp12 = Fp[w]/(w^12 - 2 w^6 + 2), in which u = w^6 - 1, so w^6 = u + 1 and the map
    (x', y') -> (x'/w^2, y'/w^3) carries E'(Fp2) into E(Fp12): y^2 = x^3 + 4;
  * Miller's algorithm with chord and tangent lines of E(Fp12) evaluated at the G1 point,
    over the bits of |z| (z the curve parameter), vertical lines dropped;
  * since z < 0 the function f_{z,Q} is the inverse of f_{|z|,Q} up to vertical lines;
  * final exponentiation by the integer (p^12 - 1)/r, one plain power.
Elements of Fp12 are lists of 12 coefficients of w^0 .. w^11 (Python ints mod p); their byte
encoding is those 12 values, 48 bytes little-endian each.
"""
from . import bls12_381 as ec
from .bls12_381 import INF, P, R, Z_BLS

# --- Fp2 ----------------------------------------------------------------------------------
F2_ZERO = (0, 0)
F2_ONE = (1, 0)
XI = (1, 1)                                       # u + 1, the non-residue that defines the twist


def f2_add(a, b):
    return ((a[0] + b[0]) % P, (a[1] + b[1]) % P)


def f2_sub(a, b):
    return ((a[0] - b[0]) % P, (a[1] - b[1]) % P)


def f2_neg(a):
    return ((-a[0]) % P, (-a[1]) % P)


def f2_mul(a, b):
    return ((a[0] * b[0] - a[1] * b[1]) % P, (a[0] * b[1] + a[1] * b[0]) % P)


def f2_inv(a):
    n = (a[0] * a[0] + a[1] * a[1]) % P          # norm a * conj(a)
    if n == 0:
        raise ZeroDivisionError("inverse of 0 in Fp2")
    ni = ec.fp_inv(n)
    return (a[0] * ni % P, (-a[1]) * ni % P)


def f2_scalar(a, k):
    return (a[0] * k % P, a[1] * k % P)


# --- G2: the order-r subgroup of E'(Fp2): y^2 = x^3 + 4(u + 1) ---------------------------
B2 = f2_scalar(XI, ec.B_COEFF)
# the generator commonly used for BLS12-381 (x = x0 + x1 u, y = y0 + y1 u); the tests check that it is on the
# twist and has order r -- any such point would serve
G2_X = (0x024AA2B2F08F0A91260805272DC51051C6E47AD4FA403B02B4510B647AE3D1770BAC0326A805BBEFD48056C8C121BDB8,
        0x13E02B6052719F607DACD3A088274F65596BD0D09920B61AB5DA61BBDC7F5049334CF11213945D57E5AC7D055D042B7E)
G2_Y = (0x0CE5D527727D6E118CC9CDC6DA2E351AADFD9BAA8CBDD3A76D429A695160D12C923AC9CC3BACA289E193548608B82801,
        0x0606C4A02EA734CC32ACD2B02BC28B99CB3E287E85A763AF267492AB572E99AB3F370D275CEC1DA1AAA9075FF05F79BE)
G2 = (G2_X, G2_Y)
G2_BYTES = 192
GT_BYTES = 576


def g2_is_on_curve(q):
    if q is INF:
        return True
    x, y = q
    return f2_sub(f2_mul(y, y), f2_add(f2_mul(f2_mul(x, x), x), B2)) == F2_ZERO


def g2_neg(q):
    return INF if q is INF else (q[0], f2_neg(q[1]))


def g2_add(a, b):
    """Chord-and-tangent law on the twist (same shape as on E: the coefficient a is 0)."""
    if a is INF:
        return b
    if b is INF:
        return a
    (x1, y1), (x2, y2) = a, b
    if x1 == x2:
        if f2_add(y1, y2) == F2_ZERO:
            return INF
        lam = f2_mul(f2_scalar(f2_mul(x1, x1), 3), f2_inv(f2_scalar(y1, 2)))
    else:
        lam = f2_mul(f2_sub(y2, y1), f2_inv(f2_sub(x2, x1)))
    x3 = f2_sub(f2_sub(f2_mul(lam, lam), x1), x2)
    y3 = f2_sub(f2_mul(lam, f2_sub(x1, x3)), y1)
    return (x3, y3)


def g2_mul(k, q):
    k %= R
    acc = INF
    for bit in bin(k)[2:] if k else "":
        acc = g2_add(acc, acc)
        if bit == "1":
            acc = g2_add(acc, q)
    return acc


def g2_to_bytes(q):
    if q is INF:
        return bytes(G2_BYTES)
    (x0, x1), (y0, y1) = q
    return b"".join(v.to_bytes(48, "little") for v in (x0, x1, y0, y1))


def g2_from_bytes(b):
    assert len(b) == G2_BYTES
    v = [int.from_bytes(b[48 * i : 48 * (i + 1)], "little") for i in range(4)]
    if not any(v):
        return INF
    return ((v[0], v[1]), (v[2], v[3]))


# --- Fp12 = Fp[w] / (w^12 - 2 w^6 + 2) --------------------------------------------------
F12_ONE = [1] + [0] * 11


def f12_mul(a, b):
    t = [0] * 23
    for i, ai in enumerate(a):
        if ai:
            for j, bj in enumerate(b):
                t[i + j] += ai * bj
    for k in range(22, 11, -1):                   # w^k = 2 w^(k-6) - 2 w^(k-12)
        c = t[k]
        if c:
            t[k - 6] += 2 * c
            t[k - 12] -= 2 * c
    return [c % P for c in t[:12]]


def f12_add(a, b):
    return [(x + y) % P for x, y in zip(a, b)]


def f12_sub(a, b):
    return [(x - y) % P for x, y in zip(a, b)]


def f12_from_fp(x):
    return [x % P] + [0] * 11


def f12_from_f2(a):
    """a0 + a1 u with u = w^6 - 1."""
    out = [0] * 12
    out[0] = (a[0] - a[1]) % P
    out[6] = a[1] % P
    return out


def _poly_trim(a):
    while a and a[-1] == 0:
        a.pop()
    return a


def _poly_divmod(a, b):
    a = a[:]
    q = [0] * max(len(a) - len(b) + 1, 1)
    inv_lead = ec.fp_inv(b[-1])
    while len(a) >= len(b) and a:
        c = a[-1] * inv_lead % P
        s = len(a) - len(b)
        q[s] = c
        for i, bi in enumerate(b):
            a[s + i] = (a[s + i] - c * bi) % P
        _poly_trim(a)
    return q, a


def f12_inv(a):
    """Extended Euclid in Fp[w] against the modulus polynomial."""
    modulus = [2, 0, 0, 0, 0, 0, P - 2, 0, 0, 0, 0, 0, 1]
    r0, r1 = modulus, _poly_trim([c % P for c in a])
    if not r1:
        raise ZeroDivisionError("inverse of 0 in Fp12")
    s0, s1 = [], [1]                              # r_i = s_i * a  (mod modulus)
    while len(r1) > 1:
        q, rem = _poly_divmod(r0, r1)
        # s0 - q * s1
        prod = [0] * (len(q) + len(s1))
        for i, qi in enumerate(q):
            if qi:
                for j, sj in enumerate(s1):
                    prod[i + j] += qi * sj
        n = max(len(s0), len(prod))
        nxt = [((s0[i] if i < len(s0) else 0) - (prod[i] if i < len(prod) else 0)) % P for i in range(n)]
        r0, r1 = r1, rem
        s0, s1 = s1, _poly_trim(nxt)
        if not r1:
            raise ZeroDivisionError("not invertible")
    c = ec.fp_inv(r1[0])
    out = [x * c % P for x in s1]
    out += [0] * (12 - len(out))
    assert len(out) == 12
    return out


def f12_pow(a, e):
    result = F12_ONE
    for bit in bin(e)[2:]:
        result = f12_mul(result, result)
        if bit == "1":
            result = f12_mul(result, a)
    return result


def gt_to_bytes(a):
    return b"".join(c.to_bytes(48, "little") for c in a)


# --- the pairing --------------------------------------------------------------------------
_W = [0, 1] + [0] * 10
_W2_INV = f12_inv(f12_mul(_W, _W))
_W3_INV = f12_inv(f12_mul(f12_mul(_W, _W), _W))


def untwist(q):
    """E'(Fp2) -> E(Fp12): (x', y') -> (x'/w^2, y'/w^3)."""
    return (f12_mul(f12_from_f2(q[0]), _W2_INV), f12_mul(f12_from_f2(q[1]), _W3_INV))


def _line(a, b, at):
    """Value at the G1 point `at` of the line through a and b (the tangent when a == b) on E(Fp12), and a + b.
    a and b are never opposite here (orders are r, the loop stops before r)."""
    (x1, y1), (x2, y2) = a, b
    if x1 == x2 and y1 == y2:
        three_x2 = f12_mul(f12_from_fp(3), f12_mul(x1, x1))
        lam = f12_mul(three_x2, f12_inv(f12_add(y1, y1)))
    else:
        lam = f12_mul(f12_sub(y2, y1), f12_inv(f12_sub(x2, x1)))
    xp, yp = f12_from_fp(at[0]), f12_from_fp(at[1])
    value = f12_sub(f12_sub(yp, y1), f12_mul(lam, f12_sub(xp, x1)))
    x3 = f12_sub(f12_sub(f12_mul(lam, lam), x1), x2)
    y3 = f12_sub(f12_mul(lam, f12_sub(x1, x3)), y1)
    return value, (x3, y3)


def miller(p1, q2):
    """f_{|z|, Q}(P) for P in G1 (affine over Fp) and Q in G2 (affine over Fp2), neither the identity."""
    q = untwist(q2)
    t = q
    f = F12_ONE
    for bit in bin(abs(Z_BLS))[3:]:
        value, t = _line(t, t, p1)
        f = f12_mul(f12_mul(f, f), value)
        if bit == "1":
            value, t = _line(t, q, p1)
            f = f12_mul(f, value)
    return f


FINAL_EXPONENT = (P**12 - 1) // R


def final_exponentiation(f):
    return f12_pow(f, FINAL_EXPONENT)


def pairing_product(pairs):
    """prod_i e(P_i, Q_i): the Miller values are multiplied, inverted once (z < 0), and raised to (p^12 - 1)/r.
    Pairs with an identity on either side contribute 1."""
    f = F12_ONE
    for p1, q2 in pairs:
        if p1 is INF or q2 is INF:
            continue
        f = f12_mul(f, miller(p1, q2))
    return final_exponentiation(f12_inv(f))


def pairing(p1, q2):
    return pairing_product([(p1, q2)])


# --- Ver in pairing form (Def. 4.1, sum-form reading) -----------------------------------
def verifier_key(taus):
    """What pp holds for the verifier: H and [tau_i]H."""
    return [g2_mul(t, G2) for t in taus]


def verify(vkey, commitment, kappa, y, pi):
    """e(C - [y]G, H) * prod_i e(-pi_i, [tau_i]H - [zeta_i]H) == 1 with zeta_i = kappa_i + 1 (the grid 1..d)."""
    if len(pi) != len(kappa) or len(kappa) > len(vkey):
        return False
    lhs = ec.sub(commitment, ec.mul(y % R, ec.G1))
    pairs = [(lhs, G2)]
    for i, k in enumerate(kappa):
        pairs.append((ec.neg(pi[i]), g2_add(vkey[i], g2_neg(g2_mul(k + 1, G2)))))
    return pairing_product(pairs) == F12_ONE
