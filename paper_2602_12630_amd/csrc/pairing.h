/*
 * Host-side pairing for the public form of Ver (Def. 4.1; App. E for the bilinear map): the verifier of the
 * paper has no GPU, so this part of the library is plain C++ on the CPU and never touches the HIP runtime.
 *
 *   Fp2  = Fp[u] / (u^2 + 1)
 *   Fp12 = Fp2[w] / (w^6 - xi), xi = u + 1; six Fp2 coefficients of w^0 .. w^5
 *   G2   = the order-r subgroup of the twist E': y^2 = x^3 + 4 xi over Fp2; (x', y') -> (x'/w^2, y'/w^3) is the
 *          isomorphism onto E over Fp12
 *
 * e(P, Q) = f_{|z|,Q}(P)^(-(p^12 - 1)/r): Miller's loop over the bits of |z| on affine twist coordinates (one Fp2
 * inversion per step), each line taken times w^3, which lies in Fp4 and dies in the final exponentiation,
 *     l(P) = y_P w^3 - lambda x_P w^2 + (lambda x_T - y_T);
 * z < 0 turns the Miller value into its inverse, taken as the conjugate over Fp6 (the two differ by an element
 * that the final exponentiation kills); the final exponentiation is (p^6 - 1)(p^2 + 1) by conjugation, one
 * inversion and the p^2-power map, then a plain power by (p^4 - p^2 + 1)/r.
 */
#pragma once
#include <stdint.h>
#include <string.h>

#include <vector>

#include "g1.h"

namespace tc {
namespace pairing {

inline fp_t fp_from_mont(const uint32_t* limbs) {     /* a constant stored in Montgomery form already */
    fp_t r;
    for (int i = 0; i < 12; ++i) r.l[i] = limbs[i];
    return r;
}

inline fp_t pmul(const fp_t& a, const fp_t& b) { return fp_mul_host64(a, b); }
inline fp_t psqr(const fp_t& a) { return fp_mul_host64(a, a); }

/* ---- Fp2 ------------------------------------------------------------------------------- */
struct fp2 {
    fp_t a, b;       /* a + b u */
};
inline fp2 f2_zero() { return fp2{fe_zero<FpParams>(), fe_zero<FpParams>()}; }
inline fp2 f2_one() { return fp2{fe_one<FpParams>(), fe_zero<FpParams>()}; }
inline fp2 f2_from_fp(const fp_t& x) { return fp2{x, fe_zero<FpParams>()}; }
inline bool f2_is_zero(const fp2& x) { return fe_is_zero(x.a) && fe_is_zero(x.b); }
inline bool f2_eq(const fp2& x, const fp2& y) { return fe_eq(x.a, y.a) && fe_eq(x.b, y.b); }
inline fp2 f2_add(const fp2& x, const fp2& y) { return fp2{fp_add(x.a, y.a), fp_add(x.b, y.b)}; }
inline fp2 f2_sub(const fp2& x, const fp2& y) { return fp2{fp_sub(x.a, y.a), fp_sub(x.b, y.b)}; }
inline fp2 f2_neg(const fp2& x) { return fp2{fp_neg(x.a), fp_neg(x.b)}; }
inline fp2 f2_dbl(const fp2& x) { return fp2{fp_dbl(x.a), fp_dbl(x.b)}; }
inline fp2 f2_mul(const fp2& x, const fp2& y) {
    fp_t aa = pmul(x.a, y.a), bb = pmul(x.b, y.b);
    fp_t cross = pmul(fp_add(x.a, x.b), fp_add(y.a, y.b));
    return fp2{fp_sub(aa, bb), fp_sub(fp_sub(cross, aa), bb)};
}
inline fp2 f2_sqr(const fp2& x) {
    fp_t ab = pmul(x.a, x.b);
    return fp2{pmul(fp_add(x.a, x.b), fp_sub(x.a, x.b)), fp_dbl(ab)};
}
inline fp2 f2_scale(const fp2& x, const fp_t& k) { return fp2{pmul(x.a, k), pmul(x.b, k)}; }
inline fp2 f2_mul_xi(const fp2& x) { return fp2{fp_sub(x.a, x.b), fp_add(x.a, x.b)}; }      /* (a + b u)(1 + u) */
inline fp2 f2_inv(const fp2& x) {         /* conj / norm; 0 for 0 */
    fp_t n = fp_add(psqr(x.a), psqr(x.b));
    if (fe_is_zero(n)) return f2_zero();
    fp_t ni = fe_inv_gcd<FpParams>(n);
    return fp2{pmul(x.a, ni), fp_neg(pmul(x.b, ni))};
}

/* ---- Fp6 = Fp2[v] / (v^3 - xi), used for the inversion in Fp12 (v = w^2) ------------------- */
struct fp6 {
    fp2 c[3];
};
inline fp6 f6_mul(const fp6& x, const fp6& y) {
    fp2 t[5];
    for (int i = 0; i < 5; ++i) t[i] = f2_zero();
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j) t[i + j] = f2_add(t[i + j], f2_mul(x.c[i], y.c[j]));
    fp6 r;
    r.c[0] = f2_add(t[0], f2_mul_xi(t[3]));
    r.c[1] = f2_add(t[1], f2_mul_xi(t[4]));
    r.c[2] = t[2];
    return r;
}
inline fp6 f6_sub(const fp6& x, const fp6& y) {
    fp6 r;
    for (int i = 0; i < 3; ++i) r.c[i] = f2_sub(x.c[i], y.c[i]);
    return r;
}
inline fp6 f6_mul_v(const fp6& x) { return fp6{{f2_mul_xi(x.c[2]), x.c[0], x.c[1]}}; }
inline fp6 f6_inv(const fp6& x) {
    /* adjugate over Fp2: with A = c0^2 - xi c1 c2, B = xi c2^2 - c0 c1, C = c1^2 - c0 c2 the norm is
     * c0 A + xi (c2 B + c1 C) and the inverse (A + B v + C v^2) / norm */
    fp2 A = f2_sub(f2_sqr(x.c[0]), f2_mul_xi(f2_mul(x.c[1], x.c[2])));
    fp2 B = f2_sub(f2_mul_xi(f2_sqr(x.c[2])), f2_mul(x.c[0], x.c[1]));
    fp2 C = f2_sub(f2_sqr(x.c[1]), f2_mul(x.c[0], x.c[2]));
    fp2 n = f2_add(f2_mul(x.c[0], A), f2_mul_xi(f2_add(f2_mul(x.c[2], B), f2_mul(x.c[1], C))));
    fp2 ni = f2_inv(n);
    return fp6{{f2_mul(A, ni), f2_mul(B, ni), f2_mul(C, ni)}};
}

/* ---- Fp12 ------------------------------------------------------------------------------ */
struct fp12 {
    fp2 c[6];        /* sum c[k] w^k */
};
inline fp12 f12_one() {
    fp12 r;
    r.c[0] = f2_one();
    for (int i = 1; i < 6; ++i) r.c[i] = f2_zero();
    return r;
}
inline bool f12_eq(const fp12& x, const fp12& y) {
    bool e = true;
    for (int i = 0; i < 6; ++i) e = e && f2_eq(x.c[i], y.c[i]);
    return e;
}
inline fp12 f12_mul(const fp12& x, const fp12& y) {
    fp2 t[11];
    for (int i = 0; i < 11; ++i) t[i] = f2_zero();
    for (int i = 0; i < 6; ++i) {
        if (f2_is_zero(x.c[i])) continue;            /* the lines of the Miller loop have three non-zero terms */
        for (int j = 0; j < 6; ++j) t[i + j] = f2_add(t[i + j], f2_mul(x.c[i], y.c[j]));
    }
    fp12 r;
    for (int k = 0; k < 5; ++k) r.c[k] = f2_add(t[k], f2_mul_xi(t[k + 6]));
    r.c[5] = t[5];
    return r;
}
inline fp12 f12_sqr(const fp12& x) { return f12_mul(x, x); }
inline fp12 f12_conj(const fp12& x) {      /* the p^6-power map: w -> -w */
    fp12 r = x;
    for (int k = 1; k < 6; k += 2) r.c[k] = f2_neg(x.c[k]);
    return r;
}
inline fp12 f12_frob2(const fp12& x) {     /* the p^2-power map: coefficient of w^k times gamma^k */
    fp2 gamma{fp_from_mont(FROB2_GAMMA[0]), fp_from_mont(FROB2_GAMMA[1])};
    fp12 r = x;
    fp2 g = gamma;
    for (int k = 1; k < 6; ++k) {
        r.c[k] = f2_mul(x.c[k], g);
        g = f2_mul(g, gamma);
    }
    return r;
}
inline fp12 f12_inv(const fp12& x) {
    /* x = a + b w over Fp6 (w^2 = v): 1/x = (a - b w) / (a^2 - b^2 v) */
    fp6 a{{x.c[0], x.c[2], x.c[4]}}, b{{x.c[1], x.c[3], x.c[5]}};
    fp6 d = f6_inv(f6_sub(f6_mul(a, a), f6_mul_v(f6_mul(b, b))));
    fp6 ra = f6_mul(a, d), rb = f6_mul(b, d);
    fp12 r;
    for (int i = 0; i < 3; ++i) {
        r.c[2 * i] = ra.c[i];
        r.c[2 * i + 1] = f2_neg(rb.c[i]);
    }
    return r;
}
inline fp12 final_exponentiation(const fp12& f) {
    fp12 t = f12_mul(f12_conj(f), f12_inv(f));                   /* ^(p^6 - 1) */
    t = f12_mul(f12_frob2(t), t);                                /* ^(p^2 + 1) */
    fp12 r = f12_one();
    bool started = false;
    for (int i = HARD_EXP_LIMBS * 32 - 1; i >= 0; --i) {         /* ^((p^4 - p^2 + 1) / r) */
        if (started) r = f12_sqr(r);
        if ((HARD_EXP[i >> 5] >> (i & 31)) & 1u) {
            r = started ? f12_mul(r, t) : t;
            started = true;
        }
    }
    return r;
}

/* Three times the hard part splits over the curve parameter z:
 *     3 (p^4 - p^2 + 1) / r = (z - 1)^2 (z + p) (z^2 + p^2 - 1) + 3,
 * five powers by the 64-bit |z| and a few Frobenius maps instead of a 1268-bit power.  Since 3 does not divide
 * r, the cube of the pairing value is 1 exactly when the value is: this is what the verifier computes.  After
 * the easy part the element lies in the cyclotomic subgroup, where the inverse is the conjugate. */
inline fp12 f12_frob1(const fp12& x) {     /* the p-power map: conjugate coefficients, times gamma1^k */
    fp2 gamma{fp_from_mont(FROB1_GAMMA[0]), fp_from_mont(FROB1_GAMMA[1])};
    fp12 r;
    fp2 g = f2_one();
    for (int k = 0; k < 6; ++k) {
        fp2 cj{x.c[k].a, fp_neg(x.c[k].b)};
        r.c[k] = k ? f2_mul(cj, g) : cj;
        g = f2_mul(g, gamma);
    }
    return r;
}
inline fp12 cyclotomic_pow_z(const fp12& x) {      /* x^z for the negative curve parameter z */
    fp12 r = x;
    int top = 63;
    while (!((BLS_Z_ABS >> top) & 1ull)) --top;
    for (int i = top - 1; i >= 0; --i) {
        r = f12_sqr(r);
        if ((BLS_Z_ABS >> i) & 1ull) r = f12_mul(r, x);
    }
    return f12_conj(r);
}
inline fp12 final_exponentiation_cubed(const fp12& f) {
    fp12 t = f12_mul(f12_conj(f), f12_inv(f));                   /* ^(p^6 - 1) */
    t = f12_mul(f12_frob2(t), t);                                /* ^(p^2 + 1) */
    fp12 a = f12_mul(cyclotomic_pow_z(t), f12_conj(t));          /* t^(z - 1) */
    a = f12_mul(cyclotomic_pow_z(a), f12_conj(a));               /* t^((z - 1)^2) */
    fp12 b = f12_mul(cyclotomic_pow_z(a), f12_frob1(a));         /* a^(z + p) */
    fp12 c = f12_mul(f12_mul(cyclotomic_pow_z(cyclotomic_pow_z(b)), f12_frob2(b)), f12_conj(b));   /* b^(z^2 + p^2 - 1) */
    return f12_mul(c, f12_mul(f12_sqr(t), t));
}

/* ---- G2, affine on the twist (identity: both coordinates zero) --------------------------- */
struct g2_affine {
    fp2 x, y;
};
inline g2_affine g2_identity() { return g2_affine{f2_zero(), f2_zero()}; }
inline bool g2_is_identity(const g2_affine& q) { return f2_is_zero(q.x) && f2_is_zero(q.y); }
inline g2_affine g2_generator() {
    return g2_affine{fp2{fp_from_mont(G2_GEN[0]), fp_from_mont(G2_GEN[1])},
                     fp2{fp_from_mont(G2_GEN[2]), fp_from_mont(G2_GEN[3])}};
}
inline g2_affine g2_neg(const g2_affine& q) { return g2_affine{q.x, f2_neg(q.y)}; }
inline bool g2_on_curve(const g2_affine& q) {
    if (g2_is_identity(q)) return true;
    fp2 b = f2_mul_xi(f2_from_fp(fe_from_u32<FpParams>(4)));
    return f2_eq(f2_sqr(q.y), f2_add(f2_mul(f2_sqr(q.x), q.x), b));
}
/* a + b; *slope receives the slope of the line used (tangent or chord) when the sum is a regular one */
inline g2_affine g2_add(const g2_affine& a, const g2_affine& b, fp2* slope = nullptr) {
    if (g2_is_identity(a)) return b;
    if (g2_is_identity(b)) return a;
    fp2 lam;
    if (f2_eq(a.x, b.x)) {
        if (f2_is_zero(f2_add(a.y, b.y))) return g2_identity();
        fp2 x2 = f2_sqr(a.x);
        lam = f2_mul(f2_add(f2_dbl(x2), x2), f2_inv(f2_dbl(a.y)));
    } else {
        lam = f2_mul(f2_sub(b.y, a.y), f2_inv(f2_sub(b.x, a.x)));
    }
    if (slope) *slope = lam;
    g2_affine r;
    r.x = f2_sub(f2_sub(f2_sqr(lam), a.x), b.x);
    r.y = f2_sub(f2_mul(lam, f2_sub(a.x, r.x)), a.y);
    return r;
}
inline g2_affine g2_mul(const uint32_t* k, int nbits, const g2_affine& q) {
    g2_affine acc = g2_identity();
    for (int i = nbits - 1; i >= 0; --i) {
        acc = g2_add(acc, acc);
        if ((k[i >> 5] >> (i & 31)) & 1u) acc = g2_add(acc, q);
    }
    return acc;
}
/* 192 bytes: x.a, x.b, y.a, y.b, 48 bytes little-endian each, canonical */
inline void g2_to_bytes(const g2_affine& q, uint8_t out[192]) {
    const fp_t* f[4] = {&q.x.a, &q.x.b, &q.y.a, &q.y.b};
    for (int i = 0; i < 4; ++i) {
        fp_t p = fe_to_plain(*f[i]);
        memcpy(out + 48 * i, p.l, 48);
    }
}
inline bool g2_from_bytes(const uint8_t in[192], g2_affine* q) {
    fp_t f[4];
    for (int i = 0; i < 4; ++i) {
        uint32_t w[12];
        memcpy(w, in + 48 * i, 48);
        if (!limbs_gt<12>(FpParams::MOD, w)) return false;
        f[i] = fe_from_limbs<FpParams>(w);
    }
    *q = g2_affine{fp2{f[0], f[1]}, fp2{f[2], f[3]}};
    return g2_on_curve(*q);
}

/* ---- Miller loop and pairing ------------------------------------------------------------ */
inline fp12 line_value(const fp2& lam, const g2_affine& t, const g1_affine& p) {
    fp12 l;
    for (int i = 0; i < 6; ++i) l.c[i] = f2_zero();
    l.c[0] = f2_sub(f2_mul(lam, t.x), t.y);
    l.c[2] = f2_neg(f2_scale(lam, p.x));
    l.c[3] = f2_from_fp(p.y);
    return l;
}
/* f_{|z|,Q}(P), conjugated for z < 0; P and Q not the identity */
inline fp12 miller(const g1_affine& p, const g2_affine& q) {
    g2_affine t = q;
    fp12 f = f12_one();
    int top = 63;
    while (!((BLS_Z_ABS >> top) & 1ull)) --top;
    for (int i = top - 1; i >= 0; --i) {
        fp2 lam = f2_zero();
        g2_affine t2 = g2_add(t, t, &lam);
        f = f12_mul(line_value(lam, t, p), f12_sqr(f));
        t = t2;
        if ((BLS_Z_ABS >> i) & 1ull) {
            g2_affine t3 = g2_add(t, q, &lam);
            f = f12_mul(line_value(lam, t, p), f);
            t = t3;
        }
    }
    return f12_conj(f);
}
struct pair_t {
    g1_affine p;
    g2_affine q;
};
inline fp12 miller_product(const std::vector<pair_t>& pairs) {
    fp12 f = f12_one();
    for (const pair_t& pr : pairs) {
        if (affine_is_identity(pr.p) || g2_is_identity(pr.q)) continue;
        f = f12_mul(miller(pr.p, pr.q), f);
    }
    return f;
}
/* prod_i e(P_i, Q_i); pairs with an identity contribute 1 */
inline fp12 pairing_product(const std::vector<pair_t>& pairs) { return final_exponentiation(miller_product(pairs)); }
/* whether prod_i e(P_i, Q_i) = 1, through the cube of the product */
inline bool pairing_product_is_one(const std::vector<pair_t>& pairs) {
    return f12_eq(final_exponentiation_cubed(miller_product(pairs)), f12_one());
}
/* 576 bytes: the twelve Fp coefficients of w^0 .. w^11 when u is written as w^6 - 1, 48 bytes little-endian each */
inline void gt_to_bytes(const fp12& x, uint8_t out[576]) {
    for (int k = 0; k < 6; ++k) {
        fp_t lo = fe_to_plain(fp_sub(x.c[k].a, x.c[k].b)), hi = fe_to_plain(x.c[k].b);
        memcpy(out + 48 * k, lo.l, 48);
        memcpy(out + 48 * (k + 6), hi.l, 48);
    }
}

}  // namespace pairing
}  // namespace tc
