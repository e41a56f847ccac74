/*
 * Prime-field arithmetic for BLS12-381 (App. E of the paper names the curve):
 * Fp (381-bit base field, 12 x 32-bit limbs) and Fr (255-bit scalar field,
 * 8 x 32-bit limbs), both in Montgomery form with R = 2^(32 N).
 *
 * All values handed between functions are fully reduced, in [0, q).
 * The code is plain C++ over uint32_t / uint64_t so that the same functions
 * run in HIP kernels (where the 32x32+64 products map to v_mad_u64_u32 and the
 * carry chains to v_add_co / v_addc_co) and in host code of the library.
 */
#pragma once
#include <stdint.h>
#include <string.h>

#include "constants.h"

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define TC_HD __host__ __device__ __forceinline__
/* The multi-limb products are real functions on the device (operands and result travel in
 * VGPRs): a kernel with dozens of inlined 12 x 12 limb products no longer fits the
 * instruction cache and takes minutes to compile. */
#define TC_HD_CALL __host__ __device__ __attribute__((noinline))
#else
#define TC_HD inline
#define TC_HD_CALL inline
#endif

namespace tc {

template <class P>
struct alignas(16) Fe {
    uint32_t l[P::N];
};
using fp_t = Fe<FpParams>;
using fr_t = Fe<FrParams>;

template <class P>
TC_HD Fe<P> fe_zero() {
    Fe<P> r;
#pragma unroll
    for (int i = 0; i < P::N; ++i) r.l[i] = 0;
    return r;
}
template <class P>
TC_HD Fe<P> fe_one() {                     /* Montgomery form of 1 */
    Fe<P> r;
#pragma unroll
    for (int i = 0; i < P::N; ++i) r.l[i] = P::ONE[i];
    return r;
}
template <class P>
TC_HD bool fe_is_zero(const Fe<P>& a) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < P::N; ++i) o |= a.l[i];
    return o == 0;
}
template <class P>
TC_HD bool fe_eq(const Fe<P>& a, const Fe<P>& b) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < P::N; ++i) o |= a.l[i] ^ b.l[i];
    return o == 0;
}

#if defined(__HIP_DEVICE_COMPILE__)
/* Carry chains on the device: one VALU instruction per limb, the carry / borrow travelling in
 * an SGPR pair that is an explicit operand (so the compiler may schedule freely around them). */
typedef uint64_t lanemask_t;
__device__ __forceinline__ uint32_t add_co(uint32_t a, uint32_t b, lanemask_t& c) {
    uint32_t r;
    asm("v_add_co_u32_e64 %0, %1, %2, %3" : "=v"(r), "=s"(c) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t addc_co(uint32_t a, uint32_t b, lanemask_t& c) {
    uint32_t r;
    asm("v_addc_co_u32_e64 %0, %1, %2, %3, %1" : "=v"(r), "+s"(c) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t sub_co(uint32_t a, uint32_t b, lanemask_t& c) {
    uint32_t r;
    asm("v_sub_co_u32_e64 %0, %1, %2, %3" : "=v"(r), "=s"(c) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t subb_co(uint32_t a, uint32_t b, lanemask_t& c) {
    uint32_t r;
    asm("v_subb_co_u32_e64 %0, %1, %2, %3, %1" : "=v"(r), "+s"(c) : "v"(a), "v"(b));
    return r;
}
/* per lane: mask set ? x : y */
__device__ __forceinline__ uint32_t select_mask(lanemask_t mask, uint32_t x, uint32_t y) {
    uint32_t r;
    asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(y), "v"(x), "s"(mask));
    return r;
}
#endif

/* r = a - MOD if a >= MOD else a, for a < 2 MOD given as limbs plus a carry bit */
template <class P>
TC_HD Fe<P> fe_reduce_once(const Fe<P>& a, uint32_t carry) {
#if defined(__HIP_DEVICE_COMPILE__)
    /* 2 MOD < 2^(32 N) for both fields, so callers never pass a set carry */
    (void)carry;
    Fe<P> dd, rr;
    lanemask_t bw;
    dd.l[0] = sub_co(a.l[0], P::MOD[0], bw);
#pragma unroll
    for (int i = 1; i < P::N; ++i) dd.l[i] = subb_co(a.l[i], P::MOD[i], bw);
#pragma unroll
    for (int i = 0; i < P::N; ++i) rr.l[i] = select_mask(bw, a.l[i], dd.l[i]);   /* borrow: keep a */
    return rr;
#endif
    Fe<P> d;
    uint32_t borrow = 0;
#pragma unroll
    for (int i = 0; i < P::N; ++i) {
        uint64_t t = (uint64_t)a.l[i] - P::MOD[i] - borrow;
        d.l[i] = (uint32_t)t;
        borrow = (uint32_t)(t >> 63);
    }
    /* a >= MOD  <=>  carry set, or no borrow out of the subtraction */
    bool take = carry || !borrow;
    Fe<P> r;
#pragma unroll
    for (int i = 0; i < P::N; ++i) r.l[i] = take ? d.l[i] : a.l[i];
    return r;
}

template <class P>
TC_HD Fe<P> fe_add(const Fe<P>& a, const Fe<P>& b) {
#if defined(__HIP_DEVICE_COMPILE__)
    {
        Fe<P> t;
        lanemask_t cy;
        t.l[0] = add_co(a.l[0], b.l[0], cy);
#pragma unroll
        for (int i = 1; i < P::N; ++i) t.l[i] = addc_co(a.l[i], b.l[i], cy);
        return fe_reduce_once<P>(t, 0);
    }
#endif
    Fe<P> s;
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < P::N; ++i) {
        uint64_t t = (uint64_t)a.l[i] + b.l[i] + c;
        s.l[i] = (uint32_t)t;
        c = (uint32_t)(t >> 32);
    }
    return fe_reduce_once<P>(s, c);
}

template <class P>
TC_HD Fe<P> fe_sub(const Fe<P>& a, const Fe<P>& b) {
#if defined(__HIP_DEVICE_COMPILE__)
    {
        Fe<P> t, u;
        lanemask_t bw, cy;
        t.l[0] = sub_co(a.l[0], b.l[0], bw);
#pragma unroll
        for (int i = 1; i < P::N; ++i) t.l[i] = subb_co(a.l[i], b.l[i], bw);
        u.l[0] = add_co(t.l[0], P::MOD[0], cy);
#pragma unroll
        for (int i = 1; i < P::N; ++i) u.l[i] = addc_co(t.l[i], P::MOD[i], cy);
#pragma unroll
        for (int i = 0; i < P::N; ++i) u.l[i] = select_mask(bw, u.l[i], t.l[i]);   /* borrow: take t + MOD */
        return u;
    }
#endif
    Fe<P> d;
    uint32_t borrow = 0;
#pragma unroll
    for (int i = 0; i < P::N; ++i) {
        uint64_t t = (uint64_t)a.l[i] - b.l[i] - borrow;
        d.l[i] = (uint32_t)t;
        borrow = (uint32_t)(t >> 63);
    }
    /* add MOD back when the subtraction borrowed */
    uint32_t mask = 0u - borrow;
    uint32_t c = 0;
    Fe<P> r;
#pragma unroll
    for (int i = 0; i < P::N; ++i) {
        uint64_t t = (uint64_t)d.l[i] + (P::MOD[i] & mask) + c;
        r.l[i] = (uint32_t)t;
        c = (uint32_t)(t >> 32);
    }
    return r;
}

template <class P>
TC_HD Fe<P> fe_neg(const Fe<P>& a) {
    return fe_sub<P>(fe_zero<P>(), a);
}
template <class P>
TC_HD Fe<P> fe_dbl(const Fe<P>& a) {
    return fe_add<P>(a, a);
}

/* Montgomery product a b R^-1 mod q, operand scanning with interleaved reduction.
 * Row i: t += a * b_i (each column product a_j b_i + t_j fits 64 bits; the high
 * halves are folded in by one carry chain), then t += m q with m chosen so that
 * the low limb vanishes, and t is shifted down one limb. */
template <class P>
TC_HD Fe<P> fe_mul(const Fe<P>& a, const Fe<P>& b) {
    constexpr int N = P::N;
    uint32_t t[N + 1];
#pragma unroll
    for (int j = 0; j <= N; ++j) t[j] = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        uint32_t hi[N];
        uint32_t c = 0;
        uint32_t bi = b.l[i];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            uint64_t uv = (uint64_t)a.l[j] * bi + t[j];
            uint64_t s = (uint64_t)(uint32_t)uv + (j ? hi[j - 1] : 0u) + c;
            hi[j] = (uint32_t)(uv >> 32);
            t[j] = (uint32_t)s;
            c = (uint32_t)(s >> 32);
        }
        {
            uint64_t s = (uint64_t)t[N] + hi[N - 1] + c;
            t[N] = (uint32_t)s;
            /* s >> 32 is 0: the running value stays below 2 q R */
        }
        uint32_t m = t[0] * P::INV;
        c = 0;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            uint64_t uv = (uint64_t)m * P::MOD[j] + t[j];
            uint32_t lo = (uint32_t)uv;
            if (j > 0) {
                uint64_t s = (uint64_t)lo + hi[j - 1] + c;
                t[j - 1] = (uint32_t)s;
                c = (uint32_t)(s >> 32);
            }
            hi[j] = (uint32_t)(uv >> 32);
        }
        {
            uint64_t s = (uint64_t)t[N] + hi[N - 1] + c;
            t[N - 1] = (uint32_t)s;
            t[N] = (uint32_t)(s >> 32);
        }
    }
    Fe<P> r;
#pragma unroll
    for (int j = 0; j < N; ++j) r.l[j] = t[j];
    return fe_reduce_once<P>(r, t[N]);
}

#if defined(__HIP_DEVICE_COMPILE__)
/* Device form of the same product: product scanning (column by column) with one
 * 96-bit accumulator.  Each limb product is one v_mad_u64_u32 into the low 64 bits
 * plus one v_addc_co_u32 of its carry into the third word; the modulus limbs sit
 * in scalar registers.  Column k collects a_i b_{k-i} and m_i q_{k-i}; m_k is
 * chosen so that the column's low word vanishes. */
/* The carry of a multiply-add travels in an SGPR pair, and an addition that consumes it right after it was
 * written has to wait for it (the compiler pads with s_nop); the product loops therefore add the carry of one limb
 * product while the next one is under way (`flush` adds the last one before the column is shifted).  Measured
 * against adding every carry at once: a product of a wave alone on its SIMD 2.3 -> 1.9 us, the accumulation
 * kernels 2.5 % faster, a lone flat commitment 2.87 -> 2.58 ms. */
struct Acc96P {
    uint64_t lo;
    uint32_t hi;
    uint64_t pending;
    bool has;
};
__device__ __forceinline__ void carry_into(uint32_t& hi, uint64_t carry) {
    uint64_t unused;
    asm volatile("v_addc_co_u32_e64 %0, %1, 0, %0, %2" : "+v"(hi), "=s"(unused) : "s"(carry));
}
/* (volatile keeps the multiply-adds and the carry additions in the order written here; sending the unused
 * carry-out of the addition to VCC instead of an SGPR pair made the accumulation kernels 3 % slower) */
/* LATE = false adds every carry at once, in an order the compiler is free to choose: the 8-limb products of the
 * interpolation kernel, eight waves to a SIMD, never wait for a carry and ran 6 % faster that way (242 against
 * 256 ms for the 512 x 4096 tensor); the 12-limb products of kernels with three waves to a SIMD take it late. */
template <bool LATE>
__device__ __forceinline__ void macp_vv(Acc96P& A, uint32_t a, uint32_t b) {
    uint64_t carry;
    if (LATE) {
        asm volatile("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(A.lo), "=s"(carry) : "v"(a), "v"(b));
        if (A.has) carry_into(A.hi, A.pending);
        A.pending = carry;
        A.has = true;
    } else {
        uint64_t unused;
        asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(A.lo), "=s"(carry) : "v"(a), "v"(b));
        asm("v_addc_co_u32_e64 %0, %1, 0, %0, %2" : "+v"(A.hi), "=s"(unused) : "s"(carry));
    }
}
template <bool LATE>
__device__ __forceinline__ void macp_vs(Acc96P& A, uint32_t a, uint32_t b) {
    uint64_t carry;
    if (LATE) {
        asm volatile("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(A.lo), "=s"(carry) : "v"(a), "s"(b));
        if (A.has) carry_into(A.hi, A.pending);
        A.pending = carry;
        A.has = true;
    } else {
        uint64_t unused;
        asm("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(A.lo), "=s"(carry) : "v"(a), "s"(b));
        asm("v_addc_co_u32_e64 %0, %1, 0, %0, %2" : "+v"(A.hi), "=s"(unused) : "s"(carry));
    }
}
__device__ __forceinline__ void flush(Acc96P& A) {
    if (A.has) carry_into(A.hi, A.pending);
    A.has = false;
}
__device__ __forceinline__ void acc_shift(Acc96P& A) {
    flush(A);
    A.lo = (A.lo >> 32) | ((uint64_t)A.hi << 32);
    A.hi = 0;
}
template <class P>
__device__ __forceinline__ Fe<P> fe_mul_dev(const Fe<P>& a, const Fe<P>& b) {
    constexpr int N = P::N;
    Acc96P A{0, 0, 0, false};
    uint32_t m[N];
    Fe<P> r;
#pragma unroll
    for (int k = 0; k < N; ++k) {
#pragma unroll
        for (int i = 0; i <= k; ++i) macp_vv<(P::N > 8)>(A, a.l[i], b.l[k - i]);
#pragma unroll
        for (int i = 0; i < k; ++i) macp_vs<(P::N > 8)>(A, m[i], P::MOD[k - i]);
        m[k] = (uint32_t)A.lo * P::INV;
        macp_vs<(P::N > 8)>(A, m[k], P::MOD[0]);
        acc_shift(A);
    }
#pragma unroll
    for (int k = N; k < 2 * N - 1; ++k) {
#pragma unroll
        for (int i = k - N + 1; i < N; ++i) macp_vv<(P::N > 8)>(A, a.l[i], b.l[k - i]);
#pragma unroll
        for (int i = k - N + 1; i < N; ++i) macp_vs<(P::N > 8)>(A, m[i], P::MOD[k - i]);
        r.l[k - N] = (uint32_t)A.lo;
        acc_shift(A);
    }
    r.l[N - 1] = (uint32_t)A.lo;
    return fe_reduce_once<P>(r, (uint32_t)(A.lo >> 32));
}
/* Square.  a^2 = sum_j a_j 2^(32 j) (a_j 2^(32 j) + 2 (a mod 2^(32 j))), and the limbs of 2 (a mod 2^(32 j)) are
 * those of d = 2 a below position j plus, at position j, the bit c_j that a_(j-1) loses in the doubling (2 a fits
 * in the same number of limbs: the modulus leaves the top bit of the top limb free).  So column k collects
 * d_i a_j for i < j, i + j = k and, for even k, a_(k/2)^2 + c_(k/2) a_(k/2): the cross products are taken once
 * with a pre-doubled operand instead of being doubled column by column. */
template <class P>
__device__ __forceinline__ Fe<P> fe_sqr_dev(const Fe<P>& a) {
    constexpr int N = P::N;
    static_assert((P::MOD[N - 1] >> 31) == 0, "the doubled operand must fit in N limbs");
    Acc96P A{0, 0, 0, false};
    uint32_t m[N], d[N];
    Fe<P> r;
    d[0] = a.l[0] << 1;
#pragma unroll
    for (int i = 1; i < N; ++i) d[i] = __builtin_amdgcn_alignbit(a.l[i], a.l[i - 1], 31);
#pragma unroll
    for (int k = 0; k < 2 * N - 1; ++k) {
#pragma unroll
        for (int i = (k < N ? 0 : k - N + 1); i < k - i; ++i) macp_vv<(P::N > 8)>(A, d[i], a.l[k - i]);
        if ((k & 1) == 0) {
            macp_vv<(P::N > 8)>(A, a.l[k / 2], a.l[k / 2]);
            if (k) macp_vv<(P::N > 8)>(A, a.l[k / 2], a.l[k / 2 - 1] >> 31);       /* c_(k/2), formed here: registers are scarce */
        }
        if (k < N) {
#pragma unroll
            for (int i = 0; i < k; ++i) macp_vs<(P::N > 8)>(A, m[i], P::MOD[k - i]);
            m[k] = (uint32_t)A.lo * P::INV;
            macp_vs<(P::N > 8)>(A, m[k], P::MOD[0]);
        } else {
#pragma unroll
            for (int i = k - N + 1; i < N; ++i) macp_vs<(P::N > 8)>(A, m[i], P::MOD[k - i]);
            r.l[k - N] = (uint32_t)A.lo;
        }
        acc_shift(A);
    }
    r.l[N - 1] = (uint32_t)A.lo;
    return fe_reduce_once<P>(r, (uint32_t)(A.lo >> 32));
}
#endif

/* ---- Fp products on the FP64 pipe --------------------------------------------------------------
 * gfx950 issues double-precision fused multiply-adds at twice the rate of 32 x 32 + 64 integer multiply-adds,
 * and they need no carry instructions.  An Fp element is re-cut into 16 limbs of 24 bits held as doubles: a
 * limb product is below 2^48, and a whole column of the product scan -- at most 16 terms a_i b_j (the top
 * limbs of values below the modulus have 21 bits), 16 terms m_i p_j and the carry of the previous column --
 * stays below 2^53, so every fused multiply-add is exact in any rounding mode.  16 x 24 = 12 x 32 bits: the
 * Montgomery radix is the same 2^384, and the result is bit for bit that of the integer routine.
 * 512 multiply-adds replace 300 integer ones and their 300 carry additions: a full chip gets through fewer
 * products a second this way; a wave alone on its SIMD finishes a product about as fast as with the integer form
 * and a square a little sooner (tc_ctx_alu_rate measures all four). */
template <int J>
constexpr double fp_mod_limb24() {
    /* bits 24 J .. 24 J + 23 of the modulus */
    int bit = 24 * J, w = bit / 32, sh = bit % 32;
    uint64_t v = (uint64_t)FpParams::MOD[w] >> sh;
    if (sh > 8 && w + 1 < FpParams::N) v |= (uint64_t)FpParams::MOD[w + 1] << (32 - sh);
    return (double)(uint32_t)(v & 0xFFFFFFu);
}
TC_HD void fp_to_limbs24(const fp_t& a, double (&x)[16]) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        uint32_t w0 = a.l[3 * g], w1 = a.l[3 * g + 1], w2 = a.l[3 * g + 2];
        x[4 * g] = (double)(w0 & 0xFFFFFFu);
        x[4 * g + 1] = (double)(((w0 >> 24) | (w1 << 8)) & 0xFFFFFFu);
        x[4 * g + 2] = (double)(((w1 >> 16) | (w2 << 16)) & 0xFFFFFFu);
        x[4 * g + 3] = (double)(w2 >> 8);
    }
}
/* a b 2^-384 mod p from the limbs of a and b; `square` says that b is a (the cross terms are taken once, doubled) */
template <bool SQUARE>
TC_HD fp_t fp_mont_limbs24(const double (&a)[16], const double (&b)[16]) {
    const double P24[16] = {fp_mod_limb24<0>(), fp_mod_limb24<1>(), fp_mod_limb24<2>(), fp_mod_limb24<3>(),
                            fp_mod_limb24<4>(), fp_mod_limb24<5>(), fp_mod_limb24<6>(), fp_mod_limb24<7>(),
                            fp_mod_limb24<8>(), fp_mod_limb24<9>(), fp_mod_limb24<10>(), fp_mod_limb24<11>(),
                            fp_mod_limb24<12>(), fp_mod_limb24<13>(), fp_mod_limb24<14>(), fp_mod_limb24<15>()};
    const double PINV = (double)(FpParams::INV & 0xFFFFFFu);       /* -p^-1 mod 2^24 */
    const double DOWN = 0x1p-24, UP = 0x1p24;
    double m[16];
    double a2[16];
    if (SQUARE) {
#pragma unroll
        for (int i = 0; i < 16; ++i) a2[i] = a[i] + a[i];
    }
    uint32_t r[16];
    double carry = 0.0;
#pragma unroll
    for (int k = 0; k < 31; ++k) {
        double S = carry;
        const int lo = k < 16 ? 0 : k - 15, hi = k < 16 ? k : 15;
        if (SQUARE) {
#pragma unroll
            for (int i = lo; i < k - i; ++i) S = __builtin_fma(a2[i], a[k - i], S);
            if ((k & 1) == 0) S = __builtin_fma(a[k / 2], a[k / 2], S);
        } else {
#pragma unroll
            for (int i = lo; i <= hi; ++i) S = __builtin_fma(a[i], b[k - i], S);
        }
        if (k < 16) {
#pragma unroll
            for (int i = 0; i < k; ++i) S = __builtin_fma(m[i], P24[k - i], S);
            double t = __builtin_floor(S * DOWN);
            double low = __builtin_fma(-t, UP, S);                 /* S mod 2^24 */
            double q = low * PINV;
            double tq = __builtin_floor(q * DOWN);
            m[k] = __builtin_fma(-tq, UP, q);                      /* the multiple of p that clears the column's low limb */
            S = __builtin_fma(m[k], P24[0], S);
            carry = S * DOWN;
        } else {
#pragma unroll
            for (int i = lo; i <= 15; ++i) S = __builtin_fma(m[i], P24[k - i], S);
            double t = __builtin_floor(S * DOWN);
            r[k - 16] = (uint32_t)__builtin_fma(-t, UP, S);
            carry = t;
        }
    }
    r[15] = (uint32_t)carry;
    fp_t out;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        uint32_t l0 = r[4 * g], l1 = r[4 * g + 1], l2 = r[4 * g + 2], l3 = r[4 * g + 3];
        out.l[3 * g] = l0 | (l1 << 24);
        out.l[3 * g + 1] = (l1 >> 8) | (l2 << 16);
        out.l[3 * g + 2] = (l2 >> 16) | (l3 << 8);
    }
    return fe_reduce_once<FpParams>(out, 0u);
}
TC_HD fp_t fp_mul_f64(const fp_t& a, const fp_t& b) {
    double x[16], y[16];
    fp_to_limbs24(a, x);
    fp_to_limbs24(b, y);
    return fp_mont_limbs24<false>(x, y);
}
TC_HD fp_t fp_sqr_f64(const fp_t& a) {
    double x[16];
    fp_to_limbs24(a, x);
    return fp_mont_limbs24<true>(x, x);
}

/* plain (non-Montgomery) comparison a > b on limbs */
template <int N>
TC_HD bool limbs_gt(const uint32_t* a, const uint32_t* b) {
    bool gt = false, decided = false;
#pragma unroll
    for (int i = N - 1; i >= 0; --i) {
        if (!decided && a[i] != b[i]) { gt = a[i] > b[i]; decided = true; }
    }
    return gt;
}

TC_HD fp_t fp_add(const fp_t& a, const fp_t& b) { return fe_add<FpParams>(a, b); }
TC_HD fp_t fp_sub(const fp_t& a, const fp_t& b) { return fe_sub<FpParams>(a, b); }
#if defined(__HIP_DEVICE_COMPILE__)
/* The device products are real functions: operands arrive as 4-limb vectors so that the
 * calling convention keeps all 24 (16) limbs in VGPRs. */
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __attribute__((noinline)) fp_t fp_mul_call(u32x4 a0, u32x4 a1, u32x4 a2, u32x4 b0, u32x4 b1, u32x4 b2) {
    fp_t a, b;
    a.l[0] = a0.x; a.l[1] = a0.y; a.l[2] = a0.z; a.l[3] = a0.w; a.l[4] = a1.x; a.l[5] = a1.y; a.l[6] = a1.z; a.l[7] = a1.w;
    a.l[8] = a2.x; a.l[9] = a2.y; a.l[10] = a2.z; a.l[11] = a2.w;
    b.l[0] = b0.x; b.l[1] = b0.y; b.l[2] = b0.z; b.l[3] = b0.w; b.l[4] = b1.x; b.l[5] = b1.y; b.l[6] = b1.z; b.l[7] = b1.w;
    b.l[8] = b2.x; b.l[9] = b2.y; b.l[10] = b2.z; b.l[11] = b2.w;
    return fe_mul_dev<FpParams>(a, b);
}
__device__ __attribute__((noinline)) fr_t fr_mul_call(u32x4 a0, u32x4 a1, u32x4 b0, u32x4 b1) {
    fr_t a, b;
    a.l[0] = a0.x; a.l[1] = a0.y; a.l[2] = a0.z; a.l[3] = a0.w; a.l[4] = a1.x; a.l[5] = a1.y; a.l[6] = a1.z; a.l[7] = a1.w;
    b.l[0] = b0.x; b.l[1] = b0.y; b.l[2] = b0.z; b.l[3] = b0.w; b.l[4] = b1.x; b.l[5] = b1.y; b.l[6] = b1.z; b.l[7] = b1.w;
    return fe_mul_dev<FrParams>(a, b);
}
__device__ __attribute__((noinline)) fp_t fp_sqr_call(u32x4 a0, u32x4 a1, u32x4 a2) {
    fp_t a;
    a.l[0] = a0.x; a.l[1] = a0.y; a.l[2] = a0.z; a.l[3] = a0.w; a.l[4] = a1.x; a.l[5] = a1.y; a.l[6] = a1.z; a.l[7] = a1.w;
    a.l[8] = a2.x; a.l[9] = a2.y; a.l[10] = a2.z; a.l[11] = a2.w;
    return fe_sqr_dev<FpParams>(a);
}
__device__ __forceinline__ fp_t fp_sqr(const fp_t& a) {
    return fp_sqr_call(u32x4{a.l[0], a.l[1], a.l[2], a.l[3]}, u32x4{a.l[4], a.l[5], a.l[6], a.l[7]},
                       u32x4{a.l[8], a.l[9], a.l[10], a.l[11]});
}
__device__ __forceinline__ fp_t fp_mul(const fp_t& a, const fp_t& b) {
    return fp_mul_call(u32x4{a.l[0], a.l[1], a.l[2], a.l[3]}, u32x4{a.l[4], a.l[5], a.l[6], a.l[7]},
                       u32x4{a.l[8], a.l[9], a.l[10], a.l[11]}, u32x4{b.l[0], b.l[1], b.l[2], b.l[3]},
                       u32x4{b.l[4], b.l[5], b.l[6], b.l[7]}, u32x4{b.l[8], b.l[9], b.l[10], b.l[11]});
}
__device__ __forceinline__ fr_t fr_mul(const fr_t& a, const fr_t& b) {
    return fr_mul_call(u32x4{a.l[0], a.l[1], a.l[2], a.l[3]}, u32x4{a.l[4], a.l[5], a.l[6], a.l[7]},
                       u32x4{b.l[0], b.l[1], b.l[2], b.l[3]}, u32x4{b.l[4], b.l[5], b.l[6], b.l[7]});
}
/* Products for kernels whose cost is depth, not volume (the doubling chains of batch verification ran 8 % faster
 * with this form than with the integer one); a chip full of waves gets through fewer of them a second. */
__device__ __attribute__((noinline)) fp_t fp_mul_lat_call(u32x4 a0, u32x4 a1, u32x4 a2, u32x4 b0, u32x4 b1, u32x4 b2) {
    fp_t a, b;
    a.l[0] = a0.x; a.l[1] = a0.y; a.l[2] = a0.z; a.l[3] = a0.w; a.l[4] = a1.x; a.l[5] = a1.y; a.l[6] = a1.z; a.l[7] = a1.w;
    a.l[8] = a2.x; a.l[9] = a2.y; a.l[10] = a2.z; a.l[11] = a2.w;
    b.l[0] = b0.x; b.l[1] = b0.y; b.l[2] = b0.z; b.l[3] = b0.w; b.l[4] = b1.x; b.l[5] = b1.y; b.l[6] = b1.z; b.l[7] = b1.w;
    b.l[8] = b2.x; b.l[9] = b2.y; b.l[10] = b2.z; b.l[11] = b2.w;
    return fp_mul_f64(a, b);
}
__device__ __attribute__((noinline)) fp_t fp_sqr_lat_call(u32x4 a0, u32x4 a1, u32x4 a2) {
    fp_t a;
    a.l[0] = a0.x; a.l[1] = a0.y; a.l[2] = a0.z; a.l[3] = a0.w; a.l[4] = a1.x; a.l[5] = a1.y; a.l[6] = a1.z; a.l[7] = a1.w;
    a.l[8] = a2.x; a.l[9] = a2.y; a.l[10] = a2.z; a.l[11] = a2.w;
    return fp_sqr_f64(a);
}
__device__ __forceinline__ fp_t fp_mul_lat(const fp_t& a, const fp_t& b) {
    return fp_mul_lat_call(u32x4{a.l[0], a.l[1], a.l[2], a.l[3]}, u32x4{a.l[4], a.l[5], a.l[6], a.l[7]},
                           u32x4{a.l[8], a.l[9], a.l[10], a.l[11]}, u32x4{b.l[0], b.l[1], b.l[2], b.l[3]},
                           u32x4{b.l[4], b.l[5], b.l[6], b.l[7]}, u32x4{b.l[8], b.l[9], b.l[10], b.l[11]});
}
__device__ __forceinline__ fp_t fp_sqr_lat(const fp_t& a) {
    return fp_sqr_lat_call(u32x4{a.l[0], a.l[1], a.l[2], a.l[3]}, u32x4{a.l[4], a.l[5], a.l[6], a.l[7]},
                           u32x4{a.l[8], a.l[9], a.l[10], a.l[11]});
}
#elif defined(__HIPCC__)
/* host pass of hipcc: the device bodies exist only in the device pass */
__device__ fp_t fp_mul(const fp_t& a, const fp_t& b);
__device__ fp_t fp_sqr(const fp_t& a);
__device__ fr_t fr_mul(const fr_t& a, const fr_t& b);
__device__ fp_t fp_mul_lat(const fp_t& a, const fp_t& b);
__device__ fp_t fp_sqr_lat(const fp_t& a);
#endif
/* Host code multiplies in Fp on 64-bit limbs: the same Montgomery representation (R = 2^384; the bytes of an
 * element are its little-endian value either way), about four times faster on a CPU than the 32-bit limbs that
 * suit the GPU.  Used by everything the library computes on the host (set-up tables, the pairing verifier) and
 * by the CPU builds of the kernels. */
inline fp_t fp_mul_host64(const fp_t& a, const fp_t& b) {
    typedef unsigned __int128 u128;
    uint64_t q[6], x[6], y[6], t[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = 0; i < 6; ++i) q[i] = (uint64_t)FpParams::MOD[2 * i] | ((uint64_t)FpParams::MOD[2 * i + 1] << 32);
    uint64_t inv = 1;
    for (int i = 0; i < 6; ++i) inv *= 2 - q[0] * inv;       /* Newton: q[0]^-1 mod 2^64 */
    inv = 0 - inv;
    memcpy(x, a.l, 48);
    memcpy(y, b.l, 48);
    for (int i = 0; i < 6; ++i) {
        u128 c = 0;
        for (int j = 0; j < 6; ++j) {
            c += (u128)x[j] * y[i] + t[j];
            t[j] = (uint64_t)c;
            c >>= 64;
        }
        c += t[6];
        t[6] = (uint64_t)c;
        t[7] = (uint64_t)(c >> 64);
        uint64_t m = t[0] * inv;
        c = ((u128)m * q[0] + t[0]) >> 64;
        for (int j = 1; j < 6; ++j) {
            c += (u128)m * q[j] + t[j];
            t[j - 1] = (uint64_t)c;
            c >>= 64;
        }
        c += t[6];
        t[5] = (uint64_t)c;
        t[6] = t[7] + (uint64_t)(c >> 64);
    }
    uint64_t d[6];
    u128 bw = 0;
    for (int j = 0; j < 6; ++j) {                            /* t < 2 q: one conditional subtraction */
        u128 s = (u128)t[j] - q[j] - (uint64_t)bw;
        d[j] = (uint64_t)s;
        bw = (s >> 64) & 1;
    }
    bool take = t[6] != 0 || bw == 0;
    fp_t r;
    memcpy(r.l, take ? d : t, 48);
    return r;
}
#if defined(__HIPCC__)
__host__ inline fp_t fp_mul(const fp_t& a, const fp_t& b) { return fp_mul_host64(a, b); }
__host__ inline fp_t fp_sqr(const fp_t& a) { return fp_mul_host64(a, a); }
__host__ inline fr_t fr_mul(const fr_t& a, const fr_t& b) { return fe_mul<FrParams>(a, b); }
__host__ inline fp_t fp_mul_lat(const fp_t& a, const fp_t& b) { return fp_mul_host64(a, b); }
__host__ inline fp_t fp_sqr_lat(const fp_t& a) { return fp_mul_host64(a, a); }
#else
inline fp_t fp_mul(const fp_t& a, const fp_t& b) { return fp_mul_host64(a, b); }
inline fp_t fp_sqr(const fp_t& a) { return fp_mul_host64(a, a); }
inline fr_t fr_mul(const fr_t& a, const fr_t& b) { return fe_mul<FrParams>(a, b); }
inline fp_t fp_mul_lat(const fp_t& a, const fp_t& b) { return fp_mul_host64(a, b); }
inline fp_t fp_sqr_lat(const fp_t& a) { return fp_mul_host64(a, a); }
#endif
/* overloads that pick the right product for generic helpers */
TC_HD fp_t fe_mulx(const fp_t& a, const fp_t& b) { return fp_mul(a, b); }
TC_HD fr_t fe_mulx(const fr_t& a, const fr_t& b) { return fr_mul(a, b); }

template <class P>
TC_HD Fe<P> fe_sqr(const Fe<P>& a) {
    return fe_mulx(a, a);
}

template <class P>
TC_HD Fe<P> fe_from_limbs(const uint32_t* w) {   /* plain value -> Montgomery form */
    Fe<P> a, r2;
#pragma unroll
    for (int i = 0; i < P::N; ++i) { a.l[i] = w[i]; r2.l[i] = P::R2[i]; }
    return fe_mulx(a, r2);
}
template <class P>
TC_HD Fe<P> fe_to_plain(const Fe<P>& a) {        /* Montgomery form -> plain value */
    Fe<P> one = fe_zero<P>();
    one.l[0] = 1;
    return fe_mulx(a, one);
}
template <class P>
TC_HD Fe<P> fe_from_u32(uint32_t v) {
    uint32_t w[P::N];
#pragma unroll
    for (int i = 0; i < P::N; ++i) w[i] = 0;
    w[0] = v;
    return fe_from_limbs<P>(w);
}
/* signed small integer -> field element (negatives as q - |v|) */
template <class P>
TC_HD Fe<P> fe_from_i32(int32_t v) {
    Fe<P> m = fe_from_u32<P>(v < 0 ? (uint32_t)(-(int64_t)v) : (uint32_t)v);
    return v < 0 ? fe_neg<P>(m) : m;
}

/* a^(q-2) by square-and-multiply (Fermat inverse); a != 0 */
template <class P>
TC_HD Fe<P> fe_inv_fermat(const Fe<P>& a) {
    Fe<P> acc = fe_one<P>();
    for (int i = P::N * 32 - 1; i >= 0; --i) {
        acc = fe_sqr<P>(acc);
        if ((P::MOD_M2[i >> 5] >> (i & 31)) & 1u) acc = fe_mulx(acc, a);
    }
    return acc;
}

/* Inverse of a non-zero element in Montgomery form, by the binary extended Euclid
 * algorithm on the plain representative (shifts, subtractions and selects only; the same
 * 64 N steps for every input, so the lanes of a wave never diverge):
 *   invariants  a = u x,  b = v x  (mod q),  b odd;  each step: if a is odd, order the
 *   pair so that a >= b and subtract (a, u) -= (b, v); then halve a and u.
 * After 2 len(q) - 1 steps a = 0 and b = 1, so v = x^-1; x = a_mont = A R, and
 * (A R)^-1 R^3 / R = A^-1 R restores the Montgomery form. */
template <class P>
TC_HD Fe<P> fe_inv(const Fe<P>& x) {
    constexpr int N = P::N;
    uint32_t a[N], b[N], u[N], v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) { a[i] = x.l[i]; b[i] = P::MOD[i]; u[i] = 0; v[i] = 0; }
    u[0] = 1;
#if defined(__HIP_DEVICE_COMPILE__)
    for (int it = 0; it < 64 * N; ++it) {
        /* lanes where a is odd and a < b exchange (a, u) with (b, v) */
        lanemask_t lt, odd;
        (void)sub_co(a[0], b[0], lt);
#pragma unroll
        for (int i = 1; i < N; ++i) (void)subb_co(a[i], b[i], lt);
        asm("v_cmp_ne_u32_e64 %0, 0, %1" : "=s"(odd) : "v"(a[0] & 1u));
        lanemask_t swap = lt & odd;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            uint32_t na = select_mask(swap, b[i], a[i]);
            b[i] = select_mask(swap, a[i], b[i]);
            a[i] = na;
            uint32_t nu = select_mask(swap, v[i], u[i]);
            v[i] = select_mask(swap, u[i], v[i]);
            u[i] = nu;
        }
        /* odd lanes: a -= b (no borrow now), u = u - v mod q */
        uint32_t d[N], w[N], w2[N];
        lanemask_t bw, bu, cy;
        d[0] = sub_co(a[0], b[0], bw);
#pragma unroll
        for (int i = 1; i < N; ++i) d[i] = subb_co(a[i], b[i], bw);
        w[0] = sub_co(u[0], v[0], bu);
#pragma unroll
        for (int i = 1; i < N; ++i) w[i] = subb_co(u[i], v[i], bu);
        w2[0] = add_co(w[0], P::MOD[0], cy);
#pragma unroll
        for (int i = 1; i < N; ++i) w2[i] = addc_co(w[i], P::MOD[i], cy);
        lanemask_t fix = bu & odd;          /* take w + q */
        lanemask_t plain = odd & ~bu;       /* take w */
#pragma unroll
        for (int i = 0; i < N; ++i) {
            a[i] = select_mask(odd, d[i], a[i]);
            u[i] = select_mask(fix, w2[i], select_mask(plain, w[i], u[i]));
        }
        /* halve a; halve u modulo q */
        lanemask_t uodd;
        asm("v_cmp_ne_u32_e64 %0, 0, %1" : "=s"(uodd) : "v"(u[0] & 1u));
        uint32_t h[N];
        h[0] = add_co(u[0], P::MOD[0], cy);
#pragma unroll
        for (int i = 1; i < N; ++i) h[i] = addc_co(u[i], P::MOD[i], cy);
        uint32_t top = select_mask(cy & uodd, 1u, 0u);
#pragma unroll
        for (int i = 0; i < N; ++i) u[i] = select_mask(uodd, h[i], u[i]);
#pragma unroll
        for (int i = 0; i < N - 1; ++i) {
            a[i] = __builtin_amdgcn_alignbit(a[i + 1], a[i], 1);
            u[i] = __builtin_amdgcn_alignbit(u[i + 1], u[i], 1);
        }
        a[N - 1] >>= 1;
        u[N - 1] = __builtin_amdgcn_alignbit(top, u[N - 1], 1);
    }
#else
    for (int it = 0; it < 64 * N; ++it) {
        uint32_t odd = 0u - (a[0] & 1u);
        /* borrow of a - b */
        uint32_t borrow = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            uint64_t t = (uint64_t)a[i] - b[i] - borrow;
            borrow = (uint32_t)(t >> 63);
        }
        uint32_t swap = odd & (0u - borrow);
#pragma unroll
        for (int i = 0; i < N; ++i) {
            uint32_t x1 = (a[i] ^ b[i]) & swap;
            a[i] ^= x1; b[i] ^= x1;
            uint32_t x2 = (u[i] ^ v[i]) & swap;
            u[i] ^= x2; v[i] ^= x2;
        }
        /* a -= b, u -= v (mod q) when a is odd */
        borrow = 0;
        uint32_t borrow_u = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            uint64_t t = (uint64_t)a[i] - (b[i] & odd) - borrow;
            a[i] = (uint32_t)t;
            borrow = (uint32_t)(t >> 63);
            uint64_t s = (uint64_t)u[i] - (v[i] & odd) - borrow_u;
            u[i] = (uint32_t)s;
            borrow_u = (uint32_t)(s >> 63);
        }
        uint32_t fix = 0u - borrow_u;
        uint32_t c = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            uint64_t t = (uint64_t)u[i] + (P::MOD[i] & fix) + c;
            u[i] = (uint32_t)t;
            c = (uint32_t)(t >> 32);
        }
        /* halve a; halve u modulo q (add q first when u is odd) */
        uint32_t uodd = 0u - (u[0] & 1u);
        c = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            uint64_t t = (uint64_t)u[i] + (P::MOD[i] & uodd) + c;
            u[i] = (uint32_t)t;
            c = (uint32_t)(t >> 32);
        }
#pragma unroll
        for (int i = 0; i < N - 1; ++i) {
            a[i] = (a[i] >> 1) | (a[i + 1] << 31);
            u[i] = (u[i] >> 1) | (u[i + 1] << 31);
        }
        a[N - 1] >>= 1;
        u[N - 1] = (u[N - 1] >> 1) | (c << 31);
    }
#endif
    Fe<P> r, r3;
#pragma unroll
    for (int i = 0; i < N; ++i) { r.l[i] = v[i]; r3.l[i] = P::R3[i]; }
    return fe_mulx(r, r3);
}

/* Inverse by the binary GCD with word-sized batches of steps (Pornin, "Optimized Binary GCD for
 * Modular Inversion", 2020).  Invariants a = u x 4^T, b = v x 4^T (mod q) after T rounds.  A round
 * runs 30 halving / subtracting steps on 62-bit approximations of (a, b) (their 30 low bits, which
 * decide the parities exactly, and their 32 top bits, which decide the comparisons) while recording
 * the steps as a 2 x 2 integer matrix (f0 g0; f1 g1), then applies the matrix once to the full
 * (a, b) (exact division by 2^30, signs fixed afterwards) and to (u, v) (one Montgomery-style word
 * reduction, i.e. a division by 2^32 modulo q).  After GCD_ROUNDS rounds a = 0, b = 1 and
 * x^-1 = v 4^GCD_ROUNDS; further rounds change nothing.  The final product with
 * GCD_FIX = 4^GCD_ROUNDS R^3 restores the Montgomery form of the inverse. */
template <class P>
TC_HD Fe<P> fe_inv_gcd(const Fe<P>& x) {
    constexpr int N = P::N;
    constexpr int K = 30;
    uint32_t a[N], b[N], u[N], v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) { a[i] = x.l[i]; b[i] = P::MOD[i]; u[i] = 0; v[i] = 0; }
    u[0] = 1;
    for (int round = 0; round < P::GCD_ROUNDS; ++round) {
        /* approximations: top limb index j of (a | b), then 64 bits below it */
        uint32_t ctop = a[N - 1] | b[N - 1], ahi = a[N - 1], alo = a[N - 2], bhi = b[N - 1], blo = b[N - 2];
        bool found = ctop != 0;
#pragma unroll
        for (int i = N - 2; i >= 1; --i) {
            uint32_t c = a[i] | b[i];
            bool take = !found && c != 0;
            ctop = take ? c : ctop;
            ahi = take ? a[i] : ahi; alo = take ? a[i - 1] : alo;
            bhi = take ? b[i] : bhi; blo = take ? b[i - 1] : blo;
            found = found || c != 0;
        }
        uint64_t xa, xb;
        if (!found) {                                     /* both fit in 64 bits: exact */
            xa = ((uint64_t)a[1] << 32) | a[0];
            xb = ((uint64_t)b[1] << 32) | b[0];
        } else {
            int lz = __builtin_clz(ctop);
            uint64_t ta = (((uint64_t)ahi << 32) | alo) << lz;
            uint64_t tb = (((uint64_t)bhi << 32) | blo) << lz;
            xa = (uint64_t)(a[0] & 0x3FFFFFFFu) | ((ta >> 32) << 30);
            xb = (uint64_t)(b[0] & 0x3FFFFFFFu) | ((tb >> 32) << 30);
        }
        /* when a and b fit in two limbs the `found` search above picked limb 1 only if it is
         * non-zero; with limb 1 set and everything above zero the exact values are used too */
        bool upper_zero = true;
#pragma unroll
        for (int i = 2; i < N; ++i) upper_zero = upper_zero && (a[i] | b[i]) == 0;
        if (upper_zero) {
            xa = ((uint64_t)a[1] << 32) | a[0];
            xb = ((uint64_t)b[1] << 32) | b[0];
        }
        int32_t f0 = 1, g0 = 0, f1 = 0, g1 = 1;
        for (int j = 0; j < K; ++j) {
            uint64_t odd = 0ull - (xa & 1ull);
            uint64_t swap = odd & (0ull - (uint64_t)(xa < xb));
            uint64_t t = (xa ^ xb) & swap;
            xa ^= t; xb ^= t;
            int32_t s32 = (int32_t)swap;
            int32_t tf = (f0 ^ f1) & s32, tg = (g0 ^ g1) & s32;
            f0 ^= tf; f1 ^= tf; g0 ^= tg; g1 ^= tg;
            xa -= xb & odd;
            f0 -= f1 & (int32_t)odd;
            g0 -= g1 & (int32_t)odd;
            xa >>= 1;
            f1 = (int32_t)((uint32_t)f1 << 1);          /* doubling of a possibly negative factor */
            g1 = (int32_t)((uint32_t)g1 << 1);
        }
        /* (a, b) <- (a f0 + b g0, a f1 + b g1) / 2^30, exact; then make both non-negative */
        uint32_t na[N + 1], nbv[N + 1];
        int64_t ca = 0, cb = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            ca += (int64_t)a[i] * f0 + (int64_t)b[i] * g0;
            cb += (int64_t)a[i] * f1 + (int64_t)b[i] * g1;
            na[i] = (uint32_t)ca; nbv[i] = (uint32_t)cb;
            ca >>= 32; cb >>= 32;
        }
        na[N] = (uint32_t)ca; nbv[N] = (uint32_t)cb;
        bool nega = (int32_t)na[N] < 0, negb = (int32_t)nbv[N] < 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            a[i] = (na[i] >> K) | (na[i + 1] << (32 - K));
            b[i] = (nbv[i] >> K) | (nbv[i + 1] << (32 - K));
        }
        {   /* two's complement negation where needed */
            uint32_t ma = nega ? 0xFFFFFFFFu : 0u, mb = negb ? 0xFFFFFFFFu : 0u;
            uint32_t c1 = nega ? 1u : 0u, c2 = negb ? 1u : 0u;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                uint64_t t1 = (uint64_t)(a[i] ^ ma) + c1;
                a[i] = (uint32_t)t1; c1 = (uint32_t)(t1 >> 32);
                uint64_t t2 = (uint64_t)(b[i] ^ mb) + c2;
                b[i] = (uint32_t)t2; c2 = (uint32_t)(t2 >> 32);
            }
            if (nega) { f0 = -f0; g0 = -g0; }
            if (negb) { f1 = -f1; g1 = -g1; }
        }
        /* (u, v) <- (u f0 + v g0, u f1 + v g1) / 2^32 mod q */
        uint32_t nu[N + 1], nv[N + 1];
        int64_t cu = 0, cv = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            cu += (int64_t)u[i] * f0 + (int64_t)v[i] * g0;
            cv += (int64_t)u[i] * f1 + (int64_t)v[i] * g1;
            nu[i] = (uint32_t)cu; nv[i] = (uint32_t)cv;
            cu >>= 32; cv >>= 32;
        }
        nu[N] = (uint32_t)cu; nv[N] = (uint32_t)cv;
        uint32_t qu = nu[0] * P::INV, qv = nv[0] * P::INV;
        int64_t du = 0, dv = 0;
        /* add q * MOD; the low limb becomes zero and is dropped */
        uint64_t ku = 0, kv = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            ku += (uint64_t)qu * P::MOD[i] + nu[i];
            kv += (uint64_t)qv * P::MOD[i] + nv[i];
            if (i > 0) { u[i - 1] = (uint32_t)ku; v[i - 1] = (uint32_t)kv; }
            ku >>= 32; kv >>= 32;
        }
        /* top limb: signed high word of the combination plus the carry of the addition */
        du = (int64_t)(int32_t)nu[N] + (int64_t)ku;
        dv = (int64_t)(int32_t)nv[N] + (int64_t)kv;
        u[N - 1] = (uint32_t)du; v[N - 1] = (uint32_t)dv;
        int32_t su = (int32_t)(du >> 32), sv = (int32_t)(dv >> 32);   /* -1, 0 (value in (-q, 2q)) */
        {   /* bring into [0, q): add q when negative, subtract q when >= q */
            uint32_t t1[N], t2[N];
            uint32_t c = 0, bw = 0;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                uint64_t s1 = (uint64_t)u[i] + P::MOD[i] + c;
                t1[i] = (uint32_t)s1; c = (uint32_t)(s1 >> 32);
                uint64_t s2 = (uint64_t)u[i] - P::MOD[i] - bw;
                t2[i] = (uint32_t)s2; bw = (uint32_t)(s2 >> 63);
            }
            bool neg = su < 0, ge = !neg && !bw;
#pragma unroll
            for (int i = 0; i < N; ++i) u[i] = neg ? t1[i] : (ge ? t2[i] : u[i]);
            c = 0; bw = 0;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                uint64_t s1 = (uint64_t)v[i] + P::MOD[i] + c;
                t1[i] = (uint32_t)s1; c = (uint32_t)(s1 >> 32);
                uint64_t s2 = (uint64_t)v[i] - P::MOD[i] - bw;
                t2[i] = (uint32_t)s2; bw = (uint32_t)(s2 >> 63);
            }
            neg = sv < 0; ge = !neg && !bw;
#pragma unroll
            for (int i = 0; i < N; ++i) v[i] = neg ? t1[i] : (ge ? t2[i] : v[i]);
        }
    }
    Fe<P> r, fix;
#pragma unroll
    for (int i = 0; i < N; ++i) { r.l[i] = v[i]; fix.l[i] = P::GCD_FIX[i]; }
    return fe_mulx(r, fix);
}

TC_HD fp_t fp_dbl(const fp_t& a) { return fe_dbl<FpParams>(a); }
TC_HD fp_t fp_neg(const fp_t& a) { return fe_neg<FpParams>(a); }
TC_HD fr_t fr_add(const fr_t& a, const fr_t& b) { return fe_add<FrParams>(a, b); }
TC_HD fr_t fr_sub(const fr_t& a, const fr_t& b) { return fe_sub<FrParams>(a, b); }
TC_HD fr_t fr_neg(const fr_t& a) { return fe_neg<FrParams>(a); }

}  // namespace tc
