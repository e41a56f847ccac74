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
 * Every addition handles the exceptional inputs (identity on either side,
 * equal points, opposite points) explicitly: sums of SRS points keyed by small
 * digits, constant tensors and the batched tree reductions do reach them.
 */
#pragma once
#include "field.h"

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

/* 2 (x, y) for an affine point, tangent rule in XYZZ form */
TC_HD g1_xyzz xyzz_dbl_affine(const g1_affine& p) {
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
TC_HD g1_xyzz xyzz_dbl(const g1_xyzz& p) {
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
TC_HD g1_xyzz xyzz_madd(const g1_xyzz& a, const g1_affine& q) {
    if (affine_is_identity(q)) return a;
    if (xyzz_is_identity(a)) return xyzz_from_affine(q);
    fp_t U2 = fp_mul(q.x, a.ZZ);
    fp_t S2 = fp_mul(q.y, a.ZZZ);
    fp_t Pd = fp_sub(U2, a.X);
    fp_t Rd = fp_sub(S2, a.Y);
    if (fe_is_zero(Pd)) {
        if (fe_is_zero(Rd)) return xyzz_dbl_affine(q);
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
TC_HD g1_xyzz xyzz_add(const g1_xyzz& a, const g1_xyzz& b) {
    if (xyzz_is_identity(b)) return a;
    if (xyzz_is_identity(a)) return b;
    fp_t U1 = fp_mul(a.X, b.ZZ);
    fp_t U2 = fp_mul(b.X, a.ZZ);
    fp_t S1 = fp_mul(a.Y, b.ZZZ);
    fp_t S2 = fp_mul(b.Y, a.ZZZ);
    fp_t Pd = fp_sub(U2, U1);
    fp_t Rd = fp_sub(S2, S1);
    if (fe_is_zero(Pd)) {
        if (fe_is_zero(Rd)) return xyzz_dbl(a);
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
    return xyzz_to_affine_with_inv(p, fe_inv_gcd<FpParams>(fp_mul(p.ZZ, p.ZZZ)));
}

/* [k] P for a plain (non-Montgomery) scalar of `nbits` bits, MSB-first double-and-add */
TC_HD g1_xyzz xyzz_mul_affine(const uint32_t* k, int nbits, const g1_affine& p) {
    g1_xyzz acc = xyzz_identity();
    for (int i = nbits - 1; i >= 0; --i) {
        acc = xyzz_dbl(acc);
        if ((k[i >> 5] >> (i & 31)) & 1u) acc = xyzz_madd(acc, p);
    }
    return acc;
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
