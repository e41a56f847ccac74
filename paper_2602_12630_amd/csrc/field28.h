/*
 * A second form of Fp for the bucket accumulation: 14 signed limbs of 28 bits, Montgomery radix 2^392.
 *
 * Why: in the 12 x 32-bit form every limb product (v_mad_u64_u32) is followed by an addition that carries into the
 * third word of the column sum, and every modular addition is a carry chain with a conditional subtraction.  With
 * 28-bit limbs a whole column of the product scan -- 14 terms a_i b_j, 14 terms q_i p_j and the carry of the
 * column before -- fits a signed 64-bit accumulator, so a product is 392 multiply-adds (v_mad_i64_i32) and no carry
 * instructions, and an addition or subtraction is 14 independent limb operations: limbs may grow beyond 28 bits
 * and go negative between products, and values need not lie in [0, p).
 *
 * A value is a limb vector l with value(l) = sum_j l_j 2^(28 j), standing for value(l) 2^-392 mod p.
 *   "normal":  limbs 0..12 in [0, 2^28), limb 13 a small signed number (the sign of the value lives there);
 *              what fp28_mul / fp28_sqr / fp28_carry return.
 * Bounds (checked by the host tests on extreme operands): a product is exact as long as
 *   14 max|a_j| max|b_j| + 14 * 2^56 + 2^36 < 2^63, e.g. limbs below 2^29.5 on both sides, or 2^30 against 2^29;
 * its result lies in (a b / 2^392, a b / 2^392 + p), i.e. in (-p, 2 p) whenever |a b| < 2^392 p -- the radix
 * leaves 11 bits of room above p, so sums of a few terms never need a reduction.
 *
 * Elements of the 32-bit form (Montgomery radix 2^384, canonical) enter by a re-cut of their bits moved up by 8
 * places (value 2^8 stands for the same field element under the radix 2^392); they leave through a Montgomery step
 * of those eight bits followed by the one full reduction of the path.
 */
#pragma once
#include "field.h"

namespace tc {

struct fp28 {
    int32_t l[14];
};

static constexpr int32_t FP28_MASK = (1 << 28) - 1;

/* the limbs of a 2^8 for a canonical a: bits 28 j - 8 .. 28 j + 19 of a */
TC_HD fp28 fp28_from_fp(const fp_t& a) {
    fp28 r;
    r.l[0] = (int32_t)((a.l[0] << 8) & (uint32_t)FP28_MASK);
#pragma unroll
    for (int j = 1; j < 14; ++j) {
        const int o = 28 * j - 8, w = o >> 5, sh = o & 31;
        uint32_t lo = a.l[w], hi = w + 1 < 12 ? a.l[w + 1] : 0u;
        uint32_t v = sh ? (lo >> sh) | (hi << (32 - sh)) : lo;
        r.l[j] = (int32_t)(v & (uint32_t)FP28_MASK);
    }
    return r;
}

TC_HD fp28 fp28_one() {
    fp28 r;
#pragma unroll
    for (int j = 0; j < 14; ++j) r.l[j] = Fp28Params::ONE[j];
    return r;
}
TC_HD fp28 fp28_add(const fp28& a, const fp28& b) {
    fp28 r;
#pragma unroll
    for (int j = 0; j < 14; ++j) r.l[j] = a.l[j] + b.l[j];
    return r;
}
TC_HD fp28 fp28_sub(const fp28& a, const fp28& b) {
    fp28 r;
#pragma unroll
    for (int j = 0; j < 14; ++j) r.l[j] = a.l[j] - b.l[j];
    return r;
}
/* same value, normal limbs (limbs of up to 31 bits either sign in, 28-bit limbs and a signed top limb out) */
TC_HD fp28 fp28_carry(const fp28& a) {
    fp28 r;
    int32_t c = 0;
#pragma unroll
    for (int j = 0; j < 13; ++j) {
        int32_t s = a.l[j] + c;
        r.l[j] = s & FP28_MASK;
        c = s >> 28;                       /* arithmetic: floor */
    }
    r.l[13] = a.l[13] + c;
    return r;
}

/* a b 2^-392 (mod p) -- or a^2, or a b - c e -- with normal limbs, in (v / 2^392, v / 2^392 + p) for the integer v
 * that is reduced.  Column k of the product scan collects a_i b_(k-i) (and -c_i e_(k-i)) and q_i p_(k-i); q_k is chosen
 * so that the low 28 bits of the column vanish.  The difference of two products costs one reduction, not two; its
 * column sums must obey the bound above with both products counted. */
enum { FP28_MUL = 0, FP28_SQR = 1, FP28_MUL_SUB = 2 };
/* acc += x y.  (The compiler starts every column of the scan from zero and joins it to the carry of the column
 * before with a 64-bit addition; multiply-adds written out as one chain per column save those 26 additions and cost
 * a wait state between dependent multiply-adds: no faster with three waves per SIMD, slower with fewer.) */
TC_HD void fp28_mac(int64_t& acc, int32_t x, int32_t y) { acc += (int64_t)x * (int64_t)y; }
template <int MODE>
TC_HD fp28 fp28_mont(const fp28& a, const fp28& b, const fp28& c, const fp28& e) {
    int64_t acc = 0;
    int32_t q[14], d[14];
    fp28 r;
    if (MODE == FP28_SQR) {
#pragma unroll
        for (int i = 0; i < 14; ++i) d[i] = a.l[i] + a.l[i];        /* cross terms once, with a doubled operand */
    }
    if (MODE == FP28_MUL_SUB) {
#pragma unroll
        for (int i = 0; i < 14; ++i) d[i] = -c.l[i];
    }
#pragma unroll
    for (int k = 0; k < 27; ++k) {
        const int lo = k < 14 ? 0 : k - 13, hi = k < 14 ? k : 13;
        if (MODE == FP28_SQR) {
#pragma unroll
            for (int i = lo; i < k - i; ++i) fp28_mac(acc, d[i], a.l[k - i]);
            if ((k & 1) == 0) fp28_mac(acc, a.l[k / 2], a.l[k / 2]);
        } else {
#pragma unroll
            for (int i = lo; i <= hi; ++i) fp28_mac(acc, a.l[i], b.l[k - i]);
        }
        if (MODE == FP28_MUL_SUB) {
#pragma unroll
            for (int i = lo; i <= hi; ++i) fp28_mac(acc, d[i], e.l[k - i]);
        }
        if (k < 14) {
#pragma unroll
            for (int i = 0; i < k; ++i) fp28_mac(acc, q[i], Fp28Params::MOD[k - i]);
            q[k] = (int32_t)(((uint32_t)acc * (uint32_t)Fp28Params::NINV) & (uint32_t)FP28_MASK);
            fp28_mac(acc, q[k], Fp28Params::MOD[0]);
        } else {
#pragma unroll
            for (int i = lo; i <= 13; ++i) fp28_mac(acc, q[i], Fp28Params::MOD[k - i]);
            r.l[k - 14] = (int32_t)((uint32_t)acc & (uint32_t)FP28_MASK);
        }
        acc >>= 28;                        /* arithmetic: the accumulator is signed */
    }
    r.l[13] = (int32_t)acc;
    return r;
}
/* expanded in place: for a kernel whose loop is a handful of products and nothing else (no operand shuffling around
 * calls, and the scheduler sees across products).  The fused difference exists in this form only: the four operands
 * of a call would not fit the 32 registers in which arguments travel. */
TC_HD fp28 fp28_mul_inline(const fp28& a, const fp28& b) { return fp28_mont<FP28_MUL>(a, b, a, a); }
TC_HD fp28 fp28_sqr_inline(const fp28& a) { return fp28_mont<FP28_SQR>(a, a, a, a); }
TC_HD fp28 fp28_mul_sub_inline(const fp28& a, const fp28& b, const fp28& c, const fp28& e) { return fp28_mont<FP28_MUL_SUB>(a, b, c, e); }

#if defined(__HIP_DEVICE_COMPILE__)
/* real functions on the device, as for the 32-bit form: operands and result travel in VGPRs */
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ fp28 fp28_unpack(i32x4 a0, i32x4 a1, i32x4 a2, i32x2 a3) {
    fp28 a;
    a.l[0] = a0.x; a.l[1] = a0.y; a.l[2] = a0.z; a.l[3] = a0.w; a.l[4] = a1.x; a.l[5] = a1.y; a.l[6] = a1.z; a.l[7] = a1.w;
    a.l[8] = a2.x; a.l[9] = a2.y; a.l[10] = a2.z; a.l[11] = a2.w; a.l[12] = a3.x; a.l[13] = a3.y;
    return a;
}
__device__ __attribute__((noinline)) fp28 fp28_mul_call(i32x4 a0, i32x4 a1, i32x4 a2, i32x2 a3, i32x4 b0, i32x4 b1, i32x4 b2, i32x2 b3) {
    return fp28_mul_inline(fp28_unpack(a0, a1, a2, a3), fp28_unpack(b0, b1, b2, b3));
}
__device__ __attribute__((noinline)) fp28 fp28_sqr_call(i32x4 a0, i32x4 a1, i32x4 a2, i32x2 a3) {
    return fp28_sqr_inline(fp28_unpack(a0, a1, a2, a3));
}
#define TC_FP28_ARGS(a) i32x4{a.l[0], a.l[1], a.l[2], a.l[3]}, i32x4{a.l[4], a.l[5], a.l[6], a.l[7]}, i32x4{a.l[8], a.l[9], a.l[10], a.l[11]}, i32x2{a.l[12], a.l[13]}
__device__ __forceinline__ fp28 fp28_mul(const fp28& a, const fp28& b) {
    return fp28_mul_call(i32x4{a.l[0], a.l[1], a.l[2], a.l[3]}, i32x4{a.l[4], a.l[5], a.l[6], a.l[7]}, i32x4{a.l[8], a.l[9], a.l[10], a.l[11]},
                         i32x2{a.l[12], a.l[13]}, i32x4{b.l[0], b.l[1], b.l[2], b.l[3]}, i32x4{b.l[4], b.l[5], b.l[6], b.l[7]},
                         i32x4{b.l[8], b.l[9], b.l[10], b.l[11]}, i32x2{b.l[12], b.l[13]});
}
__device__ __forceinline__ fp28 fp28_sqr(const fp28& a) {
    return fp28_sqr_call(i32x4{a.l[0], a.l[1], a.l[2], a.l[3]}, i32x4{a.l[4], a.l[5], a.l[6], a.l[7]}, i32x4{a.l[8], a.l[9], a.l[10], a.l[11]},
                         i32x2{a.l[12], a.l[13]});
}
#elif defined(__HIPCC__)
__device__ fp28 fp28_mul(const fp28& a, const fp28& b);
__device__ fp28 fp28_sqr(const fp28& a);
__host__ inline fp28 fp28_mul(const fp28& a, const fp28& b) { return fp28_mul_inline(a, b); }
__host__ inline fp28 fp28_sqr(const fp28& a) { return fp28_sqr_inline(a); }
#else
inline fp28 fp28_mul(const fp28& a, const fp28& b) { return fp28_mul_inline(a, b); }
inline fp28 fp28_sqr(const fp28& a) { return fp28_sqr_inline(a); }
#endif

/* 12 words of 32 bits from the bits 8 .. 391 of a non-negative value with normal limbs */
TC_HD fp_t fp28_pack_shr8(const uint32_t (&u)[14]) {
    fp_t r;
#pragma unroll
    for (int i = 0; i < 12; ++i) {
        const int o = 32 * i + 8, j = o / 28, sh = o % 28;
        uint32_t w = u[j] >> sh;
        if (j + 1 < 14) w |= u[j + 1] << (28 - sh);
        if (56 - sh < 32 && j + 2 < 14) w |= u[j + 2] << (56 - sh);
        r.l[i] = w;
    }
    return r;
}
/* fp28_from_fp undone: the element whose re-cut `a` is (no arithmetic: the limbs are slices of its bits) */
TC_HD fp_t fp28_recut_to_fp(const fp28& a) {
    uint32_t u[14];
#pragma unroll
    for (int j = 0; j < 14; ++j) u[j] = (uint32_t)a.l[j];
    return fp28_pack_shr8(u);
}
/* The canonical element of the 32-bit form (radix 2^384) for a value v with -256 p <= v < 512 p.  The two radices
 * differ by 2^8, so this is a Montgomery step of eight bits: a multiple q p with v + q p = 0 (mod 2^8), taken from
 * 256 p .. 511 p so that the sum is not negative, then the shift; (v + q p) / 2^8 < 4 p. */
TC_HD fp_t fp28_to_fp(const fp28& a) {
    int32_t q = (int32_t)((((uint32_t)a.l[0] * (uint32_t)Fp28Params::NINV) & 0xFFu) + 256u);
    uint32_t u[14];
    int64_t c = 0;
#pragma unroll
    for (int j = 0; j < 13; ++j) {
        c += (int64_t)q * (int64_t)Fp28Params::MOD[j] + (int64_t)a.l[j];
        u[j] = (uint32_t)c & (uint32_t)FP28_MASK;
        c >>= 28;
    }
    c += (int64_t)q * (int64_t)Fp28Params::MOD[13] + (int64_t)a.l[13];
    u[13] = (uint32_t)c;                   /* below 2^26 */
    fp_t r = fp28_pack_shr8(u);
    return fe_reduce_once<FpParams>(fe_reduce_once<FpParams>(fe_reduce_once<FpParams>(r, 0u), 0u), 0u);
}

/* the same as a real function on the device: for the end of a kernel whose loop must keep its registers */
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __attribute__((noinline)) fp_t fp28_to_fp_call(i32x4 a0, i32x4 a1, i32x4 a2, i32x2 a3) { return fp28_to_fp(fp28_unpack(a0, a1, a2, a3)); }
__device__ __forceinline__ fp_t fp28_to_fp_outlined(const fp28& a) { return fp28_to_fp_call(TC_FP28_ARGS(a)); }
#elif defined(__HIPCC__)
__device__ fp_t fp28_to_fp_outlined(const fp28& a);
__host__ inline fp_t fp28_to_fp_outlined(const fp28& a) { return fp28_to_fp(a); }
#else
inline fp_t fp28_to_fp_outlined(const fp28& a) { return fp28_to_fp(a); }
#endif

/* the first two limbs of that test only: no multiple of p is missed, and of the other values all but about
 * (2 K + 1) 2^-56 are told apart -- for a loop that cannot afford the registers of the full test and has a slower
 * path for whatever passes */
TC_HD bool fp28_maybe_zero(const fp28& a, uint32_t K) {
    uint32_t kk = ((uint32_t)a.l[0] * (uint32_t)Fp28Params::PINV + K) & (uint32_t)FP28_MASK;
    if (kk > 2u * K) return false;
    int32_t k = (int32_t)kk - (int32_t)K;
    int64_t c = ((int64_t)a.l[0] - (int64_t)k * (int64_t)Fp28Params::MOD[0]) >> 28;        /* the low 28 bits are zero by the choice of k */
    c += (int64_t)a.l[1] - (int64_t)k * (int64_t)Fp28Params::MOD[1];
    return ((uint32_t)c & (uint32_t)FP28_MASK) == 0;
}
TC_HD bool fp28_is_zero(const fp28& a, uint32_t K) {
    uint32_t kk = ((uint32_t)a.l[0] * (uint32_t)Fp28Params::PINV + K) & (uint32_t)FP28_MASK;
    if (kk > 2u * K) return false;
    int32_t k = (int32_t)kk - (int32_t)K;
    int64_t c = 0;
    uint32_t low = 0;
#pragma unroll
    for (int j = 0; j < 13; ++j) {
        c += (int64_t)a.l[j] - (int64_t)k * (int64_t)Fp28Params::MOD[j];
        low |= (uint32_t)c & (uint32_t)FP28_MASK;
        c >>= 28;
    }
    c += (int64_t)a.l[13] - (int64_t)k * (int64_t)Fp28Params::MOD[13];
    return low == 0 && c == 0;
}

/* R^2 / x (mod p), R = 2^384, for a canonical x != 0 of the 32-bit form: the inverse of a Montgomery representative,
 * in Montgomery form.  Binary GCD with word-sized batches of steps (Pornin, "Optimized Binary GCD for Modular
 * Inversion", 2020) on 28-bit limbs.  Invariants a = u x, b = v x (mod p), a and b non-negative.  A round runs 28
 * halving / subtracting steps on 64-bit approximations of (a, b) -- their 28 low bits, which decide the parities
 * exactly, and the 36 bits below the top bit of a | b, which decide the comparisons -- while recording the steps
 * as a 2 x 2 integer matrix, then applies the matrix once to (a, b) (an exact division by 2^28: the lowest limb of
 * the sums is zero and is dropped; a negative result is negated together with its matrix row) and to (u, v) (one
 * Montgomery step of a limb, i.e. a division by 2^28 modulo p).  u and v stay unreduced with a signed top limb:
 * a round adds at most p to their magnitude.  After 2 len(p) - 1 steps a = 0 and b = 1, so x^-1 = v; further
 * rounds change nothing.  The product with 2^1168 leaves the 28-bit form of R^2 / x.
 * Signed multiply-adds and no sign or carry bookkeeping in the updates: about 1500 vector instructions a round
 * (700 of them the 28 steps) where the 32-bit version (fe_inv_gcd, kept for Fr and the host) takes 2000; a lone
 * normalisation 114 -> 102 us. */
TC_HD fp_t fp_inv28(const fp_t& x) {
    constexpr int N = 14, K = 28;
    int32_t a[N], b[N], u[N], v[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const int o = 28 * j, w = o >> 5, sh = o & 31;
        uint32_t lo = x.l[w], hi = w + 1 < 12 ? x.l[w + 1] : 0u;
        uint32_t t = sh ? (lo >> sh) | (hi << (32 - sh)) : lo;
        a[j] = (int32_t)(t & (uint32_t)FP28_MASK);
        b[j] = Fp28Params::MOD[j];
        u[j] = 0;
        v[j] = 0;
    }
    u[0] = 1;
    for (int round = 0; round < Fp28Params::GCD_ROUNDS; ++round) {
        /* the three limbs from the highest one in which a | b has a bit, if that lies above limb 1 */
        int32_t ctop = a[N - 1] | b[N - 1];
        int32_t a2 = a[N - 1], a1 = a[N - 2], a0 = a[N - 3], b2 = b[N - 1], b1 = b[N - 2], b0 = b[N - 3];
        bool found = ctop != 0;
#pragma unroll
        for (int i = N - 2; i >= 2; --i) {
            int32_t c = a[i] | b[i];
            bool take = !found && c != 0;
            ctop = take ? c : ctop;
            a2 = take ? a[i] : a2; a1 = take ? a[i - 1] : a1; a0 = take ? a[i - 2] : a0;
            b2 = take ? b[i] : b2; b1 = take ? b[i - 1] : b1; b0 = take ? b[i - 2] : b0;
            found = found || c != 0;
        }
        uint64_t xa, xb;
        if (!found) {                                             /* both fit in 56 bits: exact */
            xa = (uint64_t)(uint32_t)a[0] | ((uint64_t)(uint32_t)a[1] << 28);
            xb = (uint64_t)(uint32_t)b[0] | ((uint64_t)(uint32_t)b[1] << 28);
        } else {
            int s = __builtin_clz((uint32_t)ctop) - 4;            /* leading zeros inside the 28-bit limb */
            uint64_t va = ((uint64_t)(uint32_t)a2 << 36) | ((uint64_t)(uint32_t)a1 << 8) | ((uint32_t)a0 >> 20);
            uint64_t vb = ((uint64_t)(uint32_t)b2 << 36) | ((uint64_t)(uint32_t)b1 << 8) | ((uint32_t)b0 >> 20);
            xa = (uint64_t)(uint32_t)a[0] | ((va >> (28 - s)) << 28);
            xb = (uint64_t)(uint32_t)b[0] | ((vb >> (28 - s)) << 28);
        }
        int32_t f0 = 1, g0 = 0, f1 = 0, g1 = 1;
        for (int j = 0; j < K; ++j) {
            bool odd = (xa & 1ull) != 0;
            bool swap = odd && xa < xb;
            uint64_t ta = swap ? xb : xa, tb = swap ? xa : xb;
            int32_t tf0 = swap ? f1 : f0, tf1 = swap ? f0 : f1, tg0 = swap ? g1 : g0, tg1 = swap ? g0 : g1;
            ta -= odd ? tb : 0ull;
            tf0 -= odd ? tf1 : 0;
            tg0 -= odd ? tg1 : 0;
            xa = ta >> 1;
            xb = tb;
            f0 = tf0;
            g0 = tg0;
            f1 = (int32_t)((uint32_t)tf1 << 1);               /* doubling of a possibly negative factor */
            g1 = (int32_t)((uint32_t)tg1 << 1);
        }
        /* (a, b) <- (a f0 + b g0, a f1 + b g1) / 2^28, exact */
        {
            int32_t na[N], nb[N];
            int64_t ca = 0, cb = 0;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                ca += (int64_t)f0 * (int64_t)a[i] + (int64_t)g0 * (int64_t)b[i];
                cb += (int64_t)f1 * (int64_t)a[i] + (int64_t)g1 * (int64_t)b[i];
                if (i > 0) {
                    na[i - 1] = (int32_t)((uint32_t)ca & (uint32_t)FP28_MASK);
                    nb[i - 1] = (int32_t)((uint32_t)cb & (uint32_t)FP28_MASK);
                }
                ca >>= 28;
                cb >>= 28;
            }
            na[N - 1] = (int32_t)ca;
            nb[N - 1] = (int32_t)cb;
            bool nega = na[N - 1] < 0, negb = nb[N - 1] < 0;
            int32_t c1 = 0, c2 = 0;
#pragma unroll
            for (int i = 0; i < N - 1; ++i) {
                int32_t t1 = (nega ? -na[i] : na[i]) + c1, t2 = (negb ? -nb[i] : nb[i]) + c2;
                a[i] = t1 & FP28_MASK;
                b[i] = t2 & FP28_MASK;
                c1 = t1 >> 28;
                c2 = t2 >> 28;
            }
            a[N - 1] = (nega ? -na[N - 1] : na[N - 1]) + c1;
            b[N - 1] = (negb ? -nb[N - 1] : nb[N - 1]) + c2;
            if (nega) { f0 = -f0; g0 = -g0; }
            if (negb) { f1 = -f1; g1 = -g1; }
        }
        /* (u, v) <- (u f0 + v g0, u f1 + v g1) / 2^28 mod p */
        {
            int64_t cu = (int64_t)f0 * (int64_t)u[0] + (int64_t)g0 * (int64_t)v[0];
            int64_t cv = (int64_t)f1 * (int64_t)u[0] + (int64_t)g1 * (int64_t)v[0];
            int32_t qu = (int32_t)(((uint32_t)cu * (uint32_t)Fp28Params::NINV) & (uint32_t)FP28_MASK);
            int32_t qv = (int32_t)(((uint32_t)cv * (uint32_t)Fp28Params::NINV) & (uint32_t)FP28_MASK);
            cu = (cu + (int64_t)qu * (int64_t)Fp28Params::MOD[0]) >> 28;
            cv = (cv + (int64_t)qv * (int64_t)Fp28Params::MOD[0]) >> 28;
            int32_t nu[N], nv[N];
#pragma unroll
            for (int i = 1; i < N; ++i) {
                cu += (int64_t)f0 * (int64_t)u[i] + (int64_t)g0 * (int64_t)v[i] + (int64_t)qu * (int64_t)Fp28Params::MOD[i];
                cv += (int64_t)f1 * (int64_t)u[i] + (int64_t)g1 * (int64_t)v[i] + (int64_t)qv * (int64_t)Fp28Params::MOD[i];
                nu[i - 1] = (int32_t)((uint32_t)cu & (uint32_t)FP28_MASK);
                nv[i - 1] = (int32_t)((uint32_t)cv & (uint32_t)FP28_MASK);
                cu >>= 28;
                cv >>= 28;
            }
            nu[N - 1] = (int32_t)cu;
            nv[N - 1] = (int32_t)cv;
#pragma unroll
            for (int i = 0; i < N; ++i) { u[i] = nu[i]; v[i] = nv[i]; }
        }
    }
    fp28 r, fix;
#pragma unroll
    for (int i = 0; i < N; ++i) { r.l[i] = v[i]; fix.l[i] = Fp28Params::INV_FIX[i]; }
    return fp28_to_fp(fp28_mul(r, fix));
}

}  // namespace tc
