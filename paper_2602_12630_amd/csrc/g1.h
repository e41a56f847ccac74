/*
 * G1 of BLS12-381, E: y^2 = x^3 + 4 over Fp (App. E of the paper: the
 * chord-and-tangent law), in the forms the kernels use:
 *
 *   affine  (x, y), Montgomery limbs; the identity is stored as (0, 0), which
 *           is not on the curve;
 *   XYZZ    (X, Y, ZZ, ZZZ) with x = X/ZZ, y = Y/ZZZ, ZZ^3 = ZZZ^2; the
 *           identity is ZZ = 0.  Accumulators live in this form: adding an
 *           affine point costs 8 multiplications + 2 squarings.
 *
 * Points are stored and handed around with coordinates in the 32-bit form of
 * the field; the group law itself computes in the carry-free 28-bit form
 * (field28.h): operands are re-cut on entry, sums and differences stay
 * unreduced, a difference of two products shares one reduction, and each
 * result coordinate is reduced once on the way out.  Values on entry are below
 * 2^389 (315 p); the comments give the bounds that the zero tests and the way
 * out rely on, in multiples of p.
 *
 * Every addition handles the exceptional inputs (identity on either side,
 * equal points, opposite points) explicitly: sums of SRS points keyed by small
 * digits, constant tensors and the batched tree reductions do reach them.
 */
#pragma once
#include "field.h"
#include "field28.h"

namespace tc {

struct g1_affine {
    fp_t x, y;
};
struct g1_xyzz {
    fp_t X, Y, ZZ, ZZZ;
};

TC_HD bool affine_is_identity(const g1_affine& p) { return fe_is_zero(p.x) && fe_is_zero(p.y); }
TC_HD g1_affine affine_identity() {
    g1_affine r;
    r.x = fe_zero<FpParams>();
    r.y = fe_zero<FpParams>();
    return r;
}
TC_HD g1_affine affine_neg(const g1_affine& p) {
    g1_affine r;
    r.x = p.x;
    r.y = fp_neg(p.y);       /* (0,0) stays (0,0) */
    return r;
}
TC_HD g1_affine affine_generator() {
    g1_affine g;
#pragma unroll
    for (int i = 0; i < 12; ++i) { g.x.l[i] = G1_GEN_X[i]; g.y.l[i] = G1_GEN_Y[i]; }
    return g;
}

TC_HD g1_xyzz xyzz_identity() {
    g1_xyzz r;
    r.X = fe_one<FpParams>();
    r.Y = fe_one<FpParams>();
    r.ZZ = fe_zero<FpParams>();
    r.ZZZ = fe_zero<FpParams>();
    return r;
}
TC_HD bool xyzz_is_identity(const g1_xyzz& p) { return fe_is_zero(p.ZZ); }
TC_HD g1_xyzz xyzz_from_affine(const g1_affine& p) {
    if (affine_is_identity(p)) return xyzz_identity();
    g1_xyzz r;
    r.X = p.x;
    r.Y = p.y;
    r.ZZ = fe_one<FpParams>();
    r.ZZZ = fe_one<FpParams>();
    return r;
}
TC_HD g1_xyzz xyzz_neg(const g1_xyzz& p) {
    g1_xyzz r = p;
    r.Y = fp_neg(p.Y);
    return r;
}

struct g1_xyzz28 {
    fp28 X, Y, ZZ, ZZZ;
};
TC_HD g1_xyzz28 xyzz28_from(const g1_xyzz& p) {
    g1_xyzz28 r;
    r.X = fp28_from_fp(p.X);
    r.Y = fp28_from_fp(p.Y);
    r.ZZ = fp28_from_fp(p.ZZ);
    r.ZZZ = fp28_from_fp(p.ZZZ);
    return r;
}
TC_HD g1_xyzz xyzz28_to(const g1_xyzz28& p) {
    g1_xyzz r;
    r.X = fp28_to_fp(p.X);
    r.Y = fp28_to_fp(p.Y);
    r.ZZ = fp28_to_fp(p.ZZ);
    r.ZZZ = fp28_to_fp(p.ZZZ);
    return r;
}

/* A running sum that stays in the 28-bit form between additions: loops convert once at the end.  `inf` says that
 * the sum is the identity (v then holds nothing).  Every case of the group law is settled here.
 *
 * The products are calls (operands and result in registers), and calls keep their order: each one is placed where
 * it ends the life of an operand, so that a caller holds about ten field elements across a call.  (Measured against
 * whole operations as real functions with the products expanded in place and the sums passed by address: the tree
 * levels and the partial-sum passes 5 to 12 % slower that way.) */
struct xyzz_acc {
    g1_xyzz28 v;
    bool inf;
    bool lone;      /* the sum is one affine point so far: X, Y are re-cuts of its coordinates, ZZ = ZZZ = 1; it leaves as it came */
};
TC_HD xyzz_acc acc_identity() {
    xyzz_acc a;
    a.v.X = fp28{};
    a.v.Y = fp28{};
    a.v.ZZ = fp28{};
    a.v.ZZZ = fp28{};
    a.inf = true;
    a.lone = false;
    return a;
}
TC_HD xyzz_acc acc_from(const g1_xyzz& p) {
    if (xyzz_is_identity(p)) return acc_identity();
    xyzz_acc a;
    a.v = xyzz28_from(p);
    a.inf = false;
    a.lone = false;
    return a;
}
TC_HD g1_xyzz acc_result(const xyzz_acc& a) {
    if (a.inf) return xyzz_identity();
    if (a.lone) {
        g1_xyzz r;
        r.X = fp28_recut_to_fp(a.v.X);
        r.Y = fp28_recut_to_fp(a.v.Y);
        r.ZZ = fe_one<FpParams>();
        r.ZZZ = fe_one<FpParams>();
        return r;
    }
    g1_xyzz r = xyzz28_to(a.v);
    if (fe_is_zero(r.ZZ)) return xyzz_identity();      /* a point of order two doubled: none on this curve */
    return r;
}

/* a <- 2 a, from (X, Y, ZZ, ZZZ) of a finite point with Y != 0, coordinates below 315 p; X, ZZ, ZZZ with normal
 * limbs, the limbs of Y (a difference of two products, or a negated coordinate) within 2^28 either way.
 * U <= 630 p, V <= 159 p, W <= 41 p, S <= 21 p, M <= 120 p, X3 in (-42 p, 7 p), Y3 in (-6 p, 4 p), ZZ3 <= 21 p, ZZZ3 <= 6 p. */
TC_HD void acc_dbl(xyzz_acc& a) {
    if (a.inf) return;
    a.lone = false;
    g1_xyzz28& p = a.v;
    fp28 U = fp28_add(p.Y, p.Y);
    fp28 V = fp28_sqr(U);
    p.ZZ = fp28_mul(V, p.ZZ);
    fp28 W = fp28_mul(U, V);
    p.ZZZ = fp28_mul(W, p.ZZZ);
    fp28 S = fp28_mul(p.X, V);
    fp28 X2 = fp28_sqr(p.X);
    fp28 M = fp28_carry(fp28_add(fp28_add(X2, X2), X2));
    p.X = fp28_carry(fp28_sub(fp28_sub(fp28_sqr(M), S), S));
    p.Y = fp28_sub(fp28_mul(M, fp28_sub(S, p.X)), fp28_mul(W, p.Y));
}

/* a <- a + q (or a - q), q affine: chord rule, tangent rule for equal points, identity for opposite ones.
 * With a below 315 p: U2, S2 <= 41 p, |P|, |R| <= 356 p, PP <= 52 p, PPP, Q <= 8 p, X3 in (-20 p, 52 p), Y3 within 12 p,
 * ZZ3 <= 8 p, ZZZ3 <= 2 p. */
TC_HD void acc_madd(xyzz_acc& a, const g1_affine& q, bool negate) {
    if (affine_is_identity(q)) return;
    if (a.inf) {
        a.v.X = fp28_from_fp(q.x);
        a.v.Y = fp28_from_fp(negate ? fp_neg(q.y) : q.y);
        a.v.ZZ = fp28_one();
        a.v.ZZZ = fp28_one();
        a.inf = false;
        a.lone = true;
        return;
    }
    a.lone = false;
    fp28 x2 = fp28_from_fp(q.x), y2 = fp28_from_fp(q.y);
    if (negate) y2 = fp28_sub(fp28{}, y2);
    fp28 Pd = fp28_sub(fp28_mul(x2, a.v.ZZ), a.v.X);
    fp28 Rd = fp28_sub(fp28_mul(y2, a.v.ZZZ), a.v.Y);
    if (fp28_is_zero(Pd, 512u)) {
        if (fp28_is_zero(Rd, 512u)) {
            a.v.X = x2;
            a.v.Y = y2;
            a.v.ZZ = fp28_one();
            a.v.ZZZ = fp28_one();
            acc_dbl(a);
        } else {
            a.inf = true;
        }
        return;
    }
    fp28 PP = fp28_sqr(Pd);
    a.v.ZZ = fp28_mul(a.v.ZZ, PP);
    fp28 PPP = fp28_mul(Pd, PP);
    fp28 Q = fp28_mul(a.v.X, PP);
    a.v.ZZZ = fp28_mul(a.v.ZZZ, PPP);
    a.v.X = fp28_carry(fp28_sub(fp28_sub(fp28_sub(fp28_sqr(Rd), PPP), Q), Q));
    a.v.Y = fp28_sub(fp28_mul(Rd, fp28_sub(Q, a.v.X)), fp28_mul(a.v.Y, PPP));
}
/* a <- a + b.  With both below 315 p: U, S <= 41 p, |P|, |R| <= 82 p, PP <= 4 p, PPP, Q <= 2 p, X3 in (-6 p, 4 p),
 * Y3 within 2 p, ZZ3, ZZZ3 <= 2 p. */
TC_HD void acc_add(xyzz_acc& a, const xyzz_acc& b) {
    if (b.inf) return;
    if (a.inf) { a = b; return; }
    a.lone = false;
    fp28 U1 = fp28_mul(a.v.X, b.v.ZZ);
    fp28 Pd = fp28_sub(fp28_mul(b.v.X, a.v.ZZ), U1);
    fp28 S1 = fp28_mul(a.v.Y, b.v.ZZZ);
    fp28 Rd = fp28_sub(fp28_mul(b.v.Y, a.v.ZZZ), S1);
    if (fp28_is_zero(Pd, 128u)) {
        if (fp28_is_zero(Rd, 128u)) acc_dbl(a);
        else a.inf = true;
        return;
    }
    a.v.ZZ = fp28_mul(a.v.ZZ, b.v.ZZ);
    a.v.ZZZ = fp28_mul(a.v.ZZZ, b.v.ZZZ);
    fp28 PP = fp28_sqr(Pd);
    a.v.ZZ = fp28_mul(a.v.ZZ, PP);
    fp28 PPP = fp28_mul(Pd, PP);
    fp28 Q = fp28_mul(U1, PP);
    a.v.ZZZ = fp28_mul(a.v.ZZZ, PPP);
    a.v.X = fp28_carry(fp28_sub(fp28_sub(fp28_sub(fp28_sqr(Rd), PPP), Q), Q));
    a.v.Y = fp28_sub(fp28_mul(Rd, fp28_sub(Q, a.v.X)), fp28_mul(S1, PPP));
}

/* a <- a + b for two finite sums, the products expanded in place and the two products of Y under one reduction: for
 * kernels whose loop is this addition and nothing else.  No case distinctions: false (a unusable) when the
 * denominator of the chord rule may be zero in the field (equal or opposite points); the caller then takes the
 * whole sum again with acc_add.  Bounds as for acc_add. */
TC_HD bool acc_add_regular_expanded(g1_xyzz28& a, const g1_xyzz28& b) {
    fp28 U1 = fp28_mul_inline(a.X, b.ZZ);
    fp28 Pd = fp28_sub(fp28_mul_inline(b.X, a.ZZ), U1);
    if (fp28_maybe_zero(Pd, 128u)) return false;
    fp28 S1 = fp28_mul_inline(a.Y, b.ZZZ);
    fp28 Rd = fp28_sub(fp28_mul_inline(b.Y, a.ZZZ), S1);
    a.ZZ = fp28_mul_inline(a.ZZ, b.ZZ);
    a.ZZZ = fp28_mul_inline(a.ZZZ, b.ZZZ);
    fp28 PP = fp28_sqr_inline(Pd);
    a.ZZ = fp28_mul_inline(a.ZZ, PP);
    fp28 PPP = fp28_mul_inline(Pd, PP);
    fp28 Q = fp28_mul_inline(U1, PP);
    a.ZZZ = fp28_mul_inline(a.ZZZ, PPP);
    a.X = fp28_carry(fp28_sub(fp28_sub(fp28_sub(fp28_sqr_inline(Rd), PPP), Q), Q));
    a.Y = fp28_mul_sub_inline(Rd, fp28_sub(Q, a.X), S1, PPP);
    return true;
}

/* the same on stored points (coordinates in the 32-bit form), one operation at a time */
TC_HD g1_xyzz xyzz_dbl_affine(const g1_affine& p) {
    xyzz_acc a = acc_identity();
    acc_madd(a, p, false);
    acc_dbl(a);
    return acc_result(a);
}
TC_HD g1_xyzz xyzz_dbl(const g1_xyzz& p) {
    xyzz_acc a = acc_from(p);
    acc_dbl(a);
    return acc_result(a);
}
TC_HD g1_xyzz xyzz_madd(const g1_xyzz& a, const g1_affine& q) {
    if (affine_is_identity(q)) return a;
    xyzz_acc A = acc_from(a);
    acc_madd(A, q, false);
    return acc_result(A);
}
TC_HD g1_xyzz xyzz_add(const g1_xyzz& a, const g1_xyzz& b) {
    if (xyzz_is_identity(b)) return a;
    if (xyzz_is_identity(a)) return b;
    xyzz_acc A = acc_from(a);
    acc_add(A, acc_from(b));
    return acc_result(A);
}

/* The same operations computed in the 32-bit form throughout, for kernels whose register budget is set by other
 * things (the cooperative sums that keep their points in LDS): slower arithmetic, about 100 registers less. */
/* 2 (x, y) for an affine point, tangent rule in XYZZ form */
TC_HD g1_xyzz xyzz_dbl_affine32(const g1_affine& p) {
    if (affine_is_identity(p) || fe_is_zero(p.y)) return xyzz_identity();
    fp_t U = fp_dbl(p.y);
    fp_t V = fp_sqr(U);
    fp_t W = fp_mul(U, V);
    fp_t S = fp_mul(p.x, V);
    fp_t X2 = fp_sqr(p.x);
    fp_t M = fp_add(fp_dbl(X2), X2);
    g1_xyzz r;
    r.X = fp_sub(fp_sub(fp_sqr(M), S), S);
    r.Y = fp_sub(fp_mul(M, fp_sub(S, r.X)), fp_mul(W, p.y));
    r.ZZ = V;
    r.ZZZ = W;
    return r;
}

/* 2 P */
TC_HD g1_xyzz xyzz_dbl32(const g1_xyzz& p) {
    if (xyzz_is_identity(p) || fe_is_zero(p.Y)) return xyzz_identity();
    fp_t U = fp_dbl(p.Y);
    fp_t V = fp_sqr(U);
    fp_t W = fp_mul(U, V);
    fp_t S = fp_mul(p.X, V);
    fp_t X2 = fp_sqr(p.X);
    fp_t M = fp_add(fp_dbl(X2), X2);
    g1_xyzz r;
    r.X = fp_sub(fp_sub(fp_sqr(M), S), S);
    r.Y = fp_sub(fp_mul(M, fp_sub(S, r.X)), fp_mul(W, p.Y));
    r.ZZ = fp_mul(V, p.ZZ);
    r.ZZZ = fp_mul(W, p.ZZZ);
    return r;
}

/* acc + q, q affine (chord rule); falls back to the tangent rule / identity when needed */
TC_HD g1_xyzz xyzz_madd32(const g1_xyzz& a, const g1_affine& q) {
    if (affine_is_identity(q)) return a;
    if (xyzz_is_identity(a)) return xyzz_from_affine(q);
    fp_t U2 = fp_mul(q.x, a.ZZ);
    fp_t S2 = fp_mul(q.y, a.ZZZ);
    fp_t Pd = fp_sub(U2, a.X);
    fp_t Rd = fp_sub(S2, a.Y);
    if (fe_is_zero(Pd)) {
        if (fe_is_zero(Rd)) return xyzz_dbl_affine32(q);
        return xyzz_identity();
    }
    fp_t PP = fp_sqr(Pd);
    fp_t PPP = fp_mul(Pd, PP);
    fp_t Q = fp_mul(a.X, PP);
    g1_xyzz r;
    r.X = fp_sub(fp_sub(fp_sub(fp_sqr(Rd), PPP), Q), Q);
    r.Y = fp_sub(fp_mul(Rd, fp_sub(Q, r.X)), fp_mul(a.Y, PPP));
    r.ZZ = fp_mul(a.ZZ, PP);
    r.ZZZ = fp_mul(a.ZZZ, PPP);
    return r;
}

/* a + b, both XYZZ */
TC_HD g1_xyzz xyzz_add32(const g1_xyzz& a, const g1_xyzz& b) {
    if (xyzz_is_identity(b)) return a;
    if (xyzz_is_identity(a)) return b;
    fp_t U1 = fp_mul(a.X, b.ZZ);
    fp_t U2 = fp_mul(b.X, a.ZZ);
    fp_t S1 = fp_mul(a.Y, b.ZZZ);
    fp_t S2 = fp_mul(b.Y, a.ZZZ);
    fp_t Pd = fp_sub(U2, U1);
    fp_t Rd = fp_sub(S2, S1);
    if (fe_is_zero(Pd)) {
        if (fe_is_zero(Rd)) return xyzz_dbl32(a);
        return xyzz_identity();
    }
    fp_t PP = fp_sqr(Pd);
    fp_t PPP = fp_mul(Pd, PP);
    fp_t Q = fp_mul(U1, PP);
    g1_xyzz r;
    r.X = fp_sub(fp_sub(fp_sub(fp_sqr(Rd), PPP), Q), Q);
    r.Y = fp_sub(fp_mul(Rd, fp_sub(Q, r.X)), fp_mul(S1, PPP));
    r.ZZ = fp_mul(fp_mul(a.ZZ, b.ZZ), PP);
    r.ZZZ = fp_mul(fp_mul(a.ZZZ, b.ZZZ), PPP);
    return r;
}

/* affine from XYZZ given inv = 1 / (ZZ * ZZZ):  1/ZZ = inv ZZZ, 1/ZZZ = inv ZZ */
TC_HD g1_affine xyzz_to_affine_with_inv(const g1_xyzz& p, const fp_t& inv) {
    if (xyzz_is_identity(p)) return affine_identity();
    g1_affine r;
    r.x = fp_mul(p.X, fp_mul(inv, p.ZZZ));
    r.y = fp_mul(p.Y, fp_mul(inv, p.ZZ));
    return r;
}
TC_HD g1_affine xyzz_to_affine(const g1_xyzz& p) {
    if (xyzz_is_identity(p)) return affine_identity();
    return xyzz_to_affine_with_inv(p, fp_inv28(fp_mul(p.ZZ, p.ZZZ)));
}

/* [k] P for a plain (non-Montgomery) scalar of `nbits` bits, MSB-first double-and-add */
TC_HD g1_xyzz xyzz_mul_affine(const uint32_t* k, int nbits, const g1_affine& p) {
    xyzz_acc acc = acc_identity();
    for (int i = nbits - 1; i >= 0; --i) {
        acc_dbl(acc);
        if ((k[i >> 5] >> (i & 31)) & 1u) acc_madd(acc, p, false);
    }
    return acc_result(acc);
}

/* Jacobian coordinates (x = X / Z^2, y = Y / Z^3; identity: Z = 0): the doubling costs two products and five
 * squarings, against six and three in XYZZ form: the form of the verifier's long doubling chains. */
struct g1_jac {
    fp_t X, Y, Z;
};
TC_HD g1_jac jac_identity() {
    g1_jac r;
    r.X = fe_one<FpParams>();
    r.Y = fe_one<FpParams>();
    r.Z = fe_zero<FpParams>();
    return r;
}
TC_HD g1_xyzz jac_to_xyzz(const g1_jac& p) {
    if (fe_is_zero(p.Z)) return xyzz_identity();
    g1_xyzz r;
    r.X = p.X;
    r.Y = p.Y;
    r.ZZ = fp_sqr(p.Z);
    r.ZZZ = fp_mul(p.Z, r.ZZ);
    return r;
}

/* canonical 96-byte encoding <-> affine Montgomery point */
TC_HD void affine_to_canonical(const g1_affine& p, uint32_t out[24]) {
    fp_t x = fe_to_plain(p.x), y = fe_to_plain(p.y);
#pragma unroll
    for (int i = 0; i < 12; ++i) { out[i] = x.l[i]; out[12 + i] = y.l[i]; }
}
TC_HD g1_affine affine_from_canonical(const uint32_t in[24]) {
    g1_affine p;
    p.x = fe_from_limbs<FpParams>(in);
    p.y = fe_from_limbs<FpParams>(in + 12);
    return p;
}

/* The map G1 -> Fr used for child commitments inside a Terkle node tensor
 * (the paper leaves it open): phi(O) = 0, phi(C) = (2 x + s(y)) mod r on the
 * canonical affine coordinates, s(y) = 1 iff y > (p-1)/2.  Returns the plain
 * (non-Montgomery) value. */
TC_HD fr_t phi_map(const g1_affine& c) {
    if (affine_is_identity(c)) return fe_zero<FrParams>();
    fp_t x = fe_to_plain(c.x), y = fe_to_plain(c.y);
    uint32_t s = limbs_gt<12>(y.l, FpParams::HALF) ? 1u : 0u;
    uint32_t v[13];
    uint32_t carry = s;
#pragma unroll
    for (int i = 0; i < 12; ++i) {
        uint64_t t = ((uint64_t)x.l[i] << 1) + carry;
        v[i] = (uint32_t)t;
        carry = (uint32_t)(t >> 32);
    }
    v[12] = carry;           /* 2x + s < 2^383: v[12] is 0 */
    /* v = lo + hi 2^256 with lo < 2^256, hi < 2^128:  lo R2 / R = lo R,  hi R3 / R = hi 2^256 R */
    fr_t lo, hi, r2, r3;
#pragma unroll
    for (int i = 0; i < 8; ++i) { lo.l[i] = v[i]; hi.l[i] = (i < 4) ? v[8 + i] : 0u; r2.l[i] = FrParams::R2[i]; r3.l[i] = FrParams::R3[i]; }
    fr_t m = fr_add(fr_mul(lo, r2), fr_mul(hi, r3));
    return fe_to_plain(m);
}

}  // namespace tc
