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

#include "constants.h"

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define TC_HD __host__ __device__ __forceinline__
#else
#define TC_HD inline
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

/* r = a - MOD if a >= MOD else a, for a < 2 MOD given as limbs plus a carry bit */
template <class P>
TC_HD Fe<P> fe_reduce_once(const Fe<P>& a, uint32_t carry) {
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

template <class P>
TC_HD Fe<P> fe_sqr(const Fe<P>& a) {
    return fe_mul<P>(a, a);
}

template <class P>
TC_HD Fe<P> fe_from_limbs(const uint32_t* w) {   /* plain value -> Montgomery form */
    Fe<P> a, r2;
#pragma unroll
    for (int i = 0; i < P::N; ++i) { a.l[i] = w[i]; r2.l[i] = P::R2[i]; }
    return fe_mul<P>(a, r2);
}
template <class P>
TC_HD Fe<P> fe_to_plain(const Fe<P>& a) {        /* Montgomery form -> plain value */
    Fe<P> one = fe_zero<P>();
    one.l[0] = 1;
    return fe_mul<P>(a, one);
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
        if ((P::MOD_M2[i >> 5] >> (i & 31)) & 1u) acc = fe_mul<P>(acc, a);
    }
    return acc;
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
TC_HD fp_t fp_mul(const fp_t& a, const fp_t& b) { return fe_mul<FpParams>(a, b); }
TC_HD fp_t fp_sqr(const fp_t& a) { return fe_sqr<FpParams>(a); }
TC_HD fp_t fp_dbl(const fp_t& a) { return fe_dbl<FpParams>(a); }
TC_HD fp_t fp_neg(const fp_t& a) { return fe_neg<FpParams>(a); }
TC_HD fr_t fr_add(const fr_t& a, const fr_t& b) { return fe_add<FrParams>(a, b); }
TC_HD fr_t fr_sub(const fr_t& a, const fr_t& b) { return fe_sub<FrParams>(a, b); }
TC_HD fr_t fr_mul(const fr_t& a, const fr_t& b) { return fe_mul<FrParams>(a, b); }
TC_HD fr_t fr_neg(const fr_t& a) { return fe_neg<FrParams>(a); }

}  // namespace tc
