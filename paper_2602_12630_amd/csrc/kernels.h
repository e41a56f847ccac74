/*
 * Kernel bodies of the library, one functor per kernel (lane = one call of
 * operator()).  Host code in tc_lib.cpp launches them through rt::launch.
 *
 * Commitment (Def. 4.1, Com) is the multi-scalar multiplication
 *     C_T = sum_i [e(T[i])] S[i]
 * over the Lagrange-basis SRS.  Scalars of quantised tensors are one signed
 * 8- or 16-bit digit, so the bucket method needs one insertion per entry:
 *     count digits -> prefix sums -> scatter point indices by bucket
 *     -> balanced segmented sums of SRS points per bucket (several passes)
 *     -> sum_k k B_k per window -> combine windows.
 * Full-width scalars (quotient values of Open, child commitments mapped into
 * Fr inside the tree) use the same engine with 8- or 16-bit signed windows, or
 * fixed-base window tables when the bases are the 16 points of a node shape.
 */
#pragma once
#include "g1.h"
#include "rt.h"

namespace tc {

enum { DT_I8 = 1, DT_I16 = 2, DT_FR = 3, DT_F16 = 4,
       DT_DIFF8 = 5, DT_DIFF16 = 6, /* internal: difference of two int8 / int16 arrays, two 9-bit signed digits */
       DT_SPLIT16 = 7, /* internal: an int16 array as two 8-bit signed digits (problems too short for 32768 buckets) */
       DT_SPLIT16M = 8, /* internal: the same two digits sharing ONE window of 128 buckets: the high digit of term i takes
                          the point i + shift of the table, which holds 2^8 times the point i */
       DT_FR128 = 9 /* internal: canonical Fr values below 2^128 (scalars split with the endomorphism): 17 windows of 8 bits */ };

struct alignas(16) fr_plain {           /* canonical (non-Montgomery) Fr value, 8 limbs */
    uint32_t l[8];
};

/* ---- small utilities ---------------------------------------------------------- */
struct Fill32 {
    uint32_t* dst;
    uint32_t value;
    TC_DEV void operator()(uint32_t t) const { dst[t] = value; }
};

/* a few words from the kernel's arguments to device memory (lane i writes word i) */
struct PokeWords {
    static constexpr uint32_t MAXW = 12;
    uint32_t* dst;
    uint32_t n;
    uint32_t w[MAXW];
    TC_DEV void operator()(uint32_t t) const { dst[t] = w[t]; }
};

/* Test hook: one field operation per lane on raw limb arrays (Montgomery representatives as they sit in
 * registers), so that the device forms of the arithmetic can be compared with big-integer arithmetic directly. */
enum { FOP_FP_MUL = 0, FOP_FP_SQR = 1, FOP_FP_MUL_F64 = 2, FOP_FP_SQR_F64 = 3, FOP_FP_INV = 4, FOP_FR_MUL = 5,
       FOP_FP_ADD = 6, FOP_FP_SUB = 7, FOP_FR_INV = 8,
       /* through the 28-bit-limb form and back: a b, a^2, (a - b)(a + b), (a - 2 b)(a - b) (limbs grown and signed) */
       FOP_FP28_MUL = 9, FOP_FP28_SQR = 10, FOP_FP28_DIFF_SUM = 11, FOP_FP28_GROWN = 12,
       FOP_FP28_MUL_SUB = 13,      /* (a - b)(a + b) - b (a - b) under one reduction */
       FOP_COUNT = 14 };
struct FieldOp {
    int op;
    const uint32_t* a;      /* 12 limbs per element (8 for the Fr operations) */
    const uint32_t* b;
    uint32_t* out;
    TC_DEV void operator()(uint32_t t) const {
        if (op == FOP_FR_MUL || op == FOP_FR_INV) {
            fr_t x, y;
#pragma unroll
            for (int i = 0; i < 8; ++i) { x.l[i] = a[8 * (uint64_t)t + i]; y.l[i] = b[8 * (uint64_t)t + i]; }
            fr_t r = op == FOP_FR_MUL ? fr_mul(x, y) : fe_inv_gcd<FrParams>(x);
#pragma unroll
            for (int i = 0; i < 8; ++i) out[8 * (uint64_t)t + i] = r.l[i];
            return;
        }
        fp_t x, y, r;
#pragma unroll
        for (int i = 0; i < 12; ++i) { x.l[i] = a[12 * (uint64_t)t + i]; y.l[i] = b[12 * (uint64_t)t + i]; }
        switch (op) {
            case FOP_FP_MUL: r = fp_mul(x, y); break;
            case FOP_FP_SQR: r = fp_sqr(x); break;
            case FOP_FP_MUL_F64: r = fp_mul_lat(x, y); break;
            case FOP_FP_SQR_F64: r = fp_sqr_lat(x); break;
            case FOP_FP_INV: r = fp_inv28(x); break;
            case FOP_FP_ADD: r = fp_add(x, y); break;
            case FOP_FP28_MUL: r = fp28_to_fp(fp28_mul(fp28_from_fp(x), fp28_from_fp(y))); break;
            case FOP_FP28_SQR: r = fp28_to_fp(fp28_sqr(fp28_from_fp(x))); break;
            case FOP_FP28_DIFF_SUM: {
                fp28 X = fp28_from_fp(x), Y = fp28_from_fp(y);
                r = fp28_to_fp(fp28_mul(fp28_sub(X, Y), fp28_add(X, Y)));
                break;
            }
            case FOP_FP28_GROWN: {
                fp28 X = fp28_from_fp(x), Y = fp28_from_fp(y);
                fp28 D = fp28_sub(X, Y);
                r = fp28_to_fp(fp28_mul(fp28_sub(D, Y), D));
                break;
            }
            case FOP_FP28_MUL_SUB: {
                fp28 X = fp28_from_fp(x), Y = fp28_from_fp(y);
                fp28 D = fp28_sub(X, Y);
                r = fp28_to_fp(fp28_mul_sub_inline(D, fp28_add(X, Y), Y, D));
                break;
            }
            default: r = fp_sub(x, y); break;
        }
#pragma unroll
        for (int i = 0; i < 12; ++i) out[12 * (uint64_t)t + i] = r.l[i];
    }
};

/* fp16 -> int16 by one float multiply, round-half-even, clamp; or pass-through copies */
struct EncodeF16 {
    const uint16_t* src;
    int16_t* dst;
    float inv_scale;
    const float* inv_scale_dev;     /* when set, the scale is read from device memory (written by the launches before) */
    TC_DEV static float half_to_float(uint16_t h) {
        uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
        uint32_t exp = (h >> 10) & 0x1Fu;
        uint32_t man = h & 0x3FFu;
        uint32_t bits;
        if (exp == 0) {
            if (man == 0) {
                bits = sign;
            } else {                         /* subnormal: normalise */
                int e = -1;
                do { man <<= 1; ++e; } while (!(man & 0x400u));
                bits = sign | ((uint32_t)(127 - 15 - e) << 23) | ((man & 0x3FFu) << 13);
            }
        } else if (exp == 31) {
            bits = sign | 0x7F800000u | (man << 13);
        } else {
            bits = sign | ((exp + 112u) << 23) | (man << 13);
        }
        float f;
        memcpy(&f, &bits, 4);
        return f;
    }
    TC_DEV static int16_t quantise(uint16_t h, float inv_scale) {
        float x = half_to_float(h);
        float y = x * inv_scale;
        float r = __builtin_rintf(y);         /* round half to even in the default mode */
        if (!(r == r)) r = 0.0f;              /* NaN -> 0 */
        if (r > 32767.0f) r = 32767.0f;
        if (r < -32767.0f) r = -32767.0f;
        return (int16_t)r;
    }
    TC_DEV void operator()(uint32_t t) const { dst[t] = quantise(src[t], inv_scale_dev ? *inv_scale_dev : inv_scale); }
};
/* the same, eight values per lane through 16-byte loads and stores (both buffers 16-byte aligned): a lane that
 * moves two bytes at a time leaves most of the HBM rate unused */
struct Words16 { uint32_t w[4]; };
struct EncodeF16x8 {
    const Words16* src;
    Words16* dst;
    float inv_scale;
    const float* inv_scale_dev;
    TC_DEV void operator()(uint32_t t) const {
        Words16 in = src[t], out;
        float s = inv_scale_dev ? *inv_scale_dev : inv_scale;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t lo = (uint16_t)EncodeF16::quantise((uint16_t)(in.w[i] & 0xFFFFu), s);
            uint32_t hi = (uint16_t)EncodeF16::quantise((uint16_t)(in.w[i] >> 16), s);
            out.w[i] = lo | (hi << 16);
        }
        dst[t] = out;
    }
};
/* Per-tensor scale of the quantisation: the largest magnitude among the finite fp16 values, then
 * inv_scale = float32(32767) / float32(amax) (0 for a tensor without a non-zero finite value).  Magnitudes of finite
 * halves order like their bit patterns without the sign bit, so the maximum is taken on 15-bit integers: a lane
 * runs over 16-byte pieces with the stride of the whole launch, a workgroup combines its lanes in LDS, and one
 * atomic maximum per workgroup lands in `result`, which the last kernel turns into the scale in place. */
TC_HD uint32_t half_magnitude_if_finite(uint32_t h) {
    uint32_t mag = h & 0x7FFFu;
    return mag < 0x7C00u ? mag : 0u;          /* exponent 31: infinities and NaNs do not count */
}
struct AbsMaxF16 {
    static constexpr int BLOCK = 1024;
    static constexpr int PHASES = 3;
    static constexpr size_t LDS_BYTES = 16;
    const uint16_t* src;
    uint64_t n;
    uint32_t groups;
    uint32_t* result;          /* zeroed before the launch */
    TC_DEV static uint32_t piece_max(const Words16& x, uint32_t best) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t a = half_magnitude_if_finite(x.w[i] & 0xFFFFu), b = half_magnitude_if_finite(x.w[i] >> 16);
            best = a > best ? a : best;
            best = b > best ? b : best;
        }
        return best;
    }
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* wmax = (uint32_t*)lds;
        if (ph == 0) {
            if (lane == 0) wmax[0] = 0;
            return;
        }
        if (ph == 2) {
            /* atomics on one address go through one after the other: a workgroup of 1024 lanes keeps them few */
            if (lane == 0 && wmax[0]) atomic_max_u32(result, wmax[0]);
            return;
        }
        uint32_t best = 0;
        /* elements before the first 16-byte boundary and after the last whole piece go one by one (workgroup 0) */
        uint64_t head = (16u - ((uintptr_t)src & 15u)) & 15u;
        head = head / 2 < n ? head / 2 : n;
        uint64_t chunks = (n - head) / 8;
        const Words16* body = (const Words16*)(src + head);
        uint64_t stride = (uint64_t)groups * BLOCK;
        uint64_t ch = (uint64_t)wg * BLOCK + lane;
        for (; ch + stride < chunks; ch += 2 * stride) {      /* two loads in flight per lane */
            Words16 x = body[ch], y = body[ch + stride];
            best = piece_max(y, piece_max(x, best));
        }
        if (ch < chunks) best = piece_max(body[ch], best);
        if (wg == 0) {
            for (uint64_t i = lane; i < head; i += BLOCK) {
                uint32_t a = half_magnitude_if_finite(src[i]);
                best = a > best ? a : best;
            }
            for (uint64_t i = head + 8 * chunks + lane; i < n; i += BLOCK) {
                uint32_t a = half_magnitude_if_finite(src[i]);
                best = a > best ? a : best;
            }
        }
        if (best) atomic_max_u32(wmax, best);
    }
};
/* the same pass over several tensors in one launch: workgroup first[j] + g is workgroup g of tensor j */
struct AbsMaxF16Batch {
    static constexpr int BLOCK = AbsMaxF16::BLOCK;
    static constexpr int PHASES = AbsMaxF16::PHASES;
    static constexpr size_t LDS_BYTES = AbsMaxF16::LDS_BYTES;
    const AbsMaxF16* jobs;
    const uint32_t* first;         /* njobs + 1 */
    uint32_t njobs;
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t lo = 0, hi = njobs;
        while (hi - lo > 1) {
            uint32_t mid = (lo + hi) / 2;
            if (first[mid] <= wg) lo = mid;
            else hi = mid;
        }
        jobs[lo].phase(ph, lane, wg - first[lo], lds);
    }
};
struct InvScaleFromAbsMax {        /* lane t: the 15-bit magnitude in result[t] becomes the float scale, in place */
    uint32_t* result;
    TC_DEV void operator()(uint32_t t) const {
        uint32_t* result = this->result + t;
        float amax = EncodeF16::half_to_float((uint16_t)*result);
        float inv = amax > 0.0f ? 32767.0f / amax : 0.0f;
        uint32_t bits;
        memcpy(&bits, &inv, 4);
        *result = bits;
    }
};
/* the same with several pieces per lane, for a launch that many tensors share (a lane first has to find its tensor) */
struct EncodeF16x8Strided {
    EncodeF16x8 one;
    uint32_t pieces, lanes;
    TC_DEV void operator()(uint32_t t) const {
        for (uint32_t i = t; i < pieces; i += lanes) one(i);
    }
};
struct Copy128 {
    const Words16* src;
    Words16* dst;
    TC_DEV void operator()(uint32_t t) const { dst[t] = src[t]; }
};
struct Copy8 {
    const uint8_t* src;
    uint8_t* dst;
    TC_DEV void operator()(uint32_t t) const { dst[t] = src[t]; }
};
struct Copy16 {
    const uint16_t* src;
    uint16_t* dst;
    TC_DEV void operator()(uint32_t t) const { dst[t] = src[t]; }
};

/* ---- signed window digits ----------------------------------------------------- */
/* Digit w of a canonical Fr value for window width c (c divides 32... c in {8,16}):
 * raw = bits + carry; raw > 2^(c-1) => digit = raw - 2^c and carry 1.  Digits lie in
 * [-(2^(c-1) - 1), 2^(c-1)].  Calls must walk w = 0, 1, .. in order and thread `carry`. */
TC_HD int32_t fr_window_digit(const uint32_t* v, int w, int c, uint32_t& carry) {
    int bit = w * c;
    uint32_t raw = (v[bit >> 5] >> (bit & 31)) & ((1u << c) - 1u);
    raw += carry;
    uint32_t half = 1u << (c - 1);
    if (raw > half) {
        carry = 1;
        return (int32_t)raw - (int32_t)(1u << c);
    }
    carry = 0;
    return (int32_t)raw;
}

TC_HD int32_t small_scalar(const void* s, int dtype, uint64_t i) {
    return (dtype == DT_I8 || dtype == DT_DIFF8) ? (int32_t)((const int8_t*)s)[i] : (int32_t)((const int16_t*)s)[i];
}
/* window digit of a small magnitude (at most 17 bits), same recoding as fr_window_digit */
TC_HD int32_t small_window_digit(uint32_t mag, int w, int c, uint32_t& carry) {
    uint32_t raw = ((mag >> (w * c)) & ((1u << c) - 1u)) + carry;
    uint32_t half = 1u << (c - 1);
    if (raw > half) {
        carry = 1;
        return (int32_t)raw - (int32_t)(1u << c);
    }
    carry = 0;
    return (int32_t)raw;
}

/* ---- MSM: count, scatter --------------------------------------------------------- */
struct MsmCount {
    const void* scalars;
    int dtype;
    int W, c;
    uint32_t nb;          /* buckets per window = 2^(c-1) */
    uint32_t* cnt;        /* W * nb counters */
    TC_DEV void operator()(uint32_t t) const {
        if (dtype == DT_FR) {
            const uint32_t* v = ((const fr_plain*)scalars)[t].l;
            uint32_t carry = 0;
            for (int w = 0; w < W; ++w) {
                int32_t d = fr_window_digit(v, w, c, carry);
                if (d) atomic_add_u32(&cnt[(uint32_t)w * nb + (uint32_t)(d < 0 ? -d : d) - 1u], 1u);
            }
        } else {
            int32_t d = small_scalar(scalars, dtype, t);
            if (d) atomic_add_u32(&cnt[(uint32_t)(d < 0 ? -d : d) - 1u], 1u);
        }
    }
};

struct MsmScatter {
    const void* scalars;
    int dtype;
    int W, c;
    uint32_t nb;
    const uint32_t* start;   /* exclusive prefix of cnt */
    uint32_t* cursor;        /* zeroed, W * nb */
    uint32_t* sorted;        /* point index | sign << 31, grouped by bucket */
    TC_DEV void put(uint32_t key, uint32_t i, bool negative) const {
        uint32_t pos = start[key] + atomic_add_u32(&cursor[key], 1u);
        sorted[pos] = i | (negative ? 0x80000000u : 0u);
    }
    TC_DEV void operator()(uint32_t t) const {
        if (dtype == DT_FR) {
            const uint32_t* v = ((const fr_plain*)scalars)[t].l;
            uint32_t carry = 0;
            for (int w = 0; w < W; ++w) {
                int32_t d = fr_window_digit(v, w, c, carry);
                if (d) put((uint32_t)w * nb + (uint32_t)(d < 0 ? -d : d) - 1u, t, d < 0);
            }
        } else {
            int32_t d = small_scalar(scalars, dtype, t);
            if (d) put((uint32_t)(d < 0 ? -d : d) - 1u, t, d < 0);
        }
    }
};

/* ---- MSM: count / scatter without global atomics (small scalars; full-width ones in 8-bit windows) ---------------- */
/* A workgroup owns a tile of consecutive terms of one problem.  CountTile builds the tile's
 * histogram in LDS and writes it as a row of the matrix M[problem][tile][key]; TileColumnScan turns
 * every column into exclusive offsets (and the per-key totals); ScatterTile reloads its row,
 * adds the global bucket starts and hands out positions with LDS atomics. */
struct TileProblem {
    const void* scalars;
    const void* sub;          /* optional subtrahend array (same element type): value = scalars[i] - sub[i] */
    uint64_t n;
    uint32_t tile;            /* terms per workgroup */
    uint32_t shift;           /* DT_SPLIT16M: digit w of term i is entered as point i + w * shift */
};
TC_HD int32_t tile_value(const TileProblem& P, int dtype, uint64_t i) {
    int32_t v = small_scalar(P.scalars, dtype, i);
    if (P.sub) v -= small_scalar(P.sub, dtype, i);
    return v;
}
/* every term i of [lo, hi) with its value v: each(i, v).  A plain int8 / int16 problem whose scalars are 16-byte
 * aligned at `lo` goes sixteen bytes per lane and step (a lane that fetches one small value per step spends its
 * time waiting for it); what is left over, and every other problem, goes term by term.  WIDE = false leaves the
 * wide path out of kernels that only ever see two-digit difference problems (it would cost them registers). */
template <int BLOCK, bool WIDE, class Each>
TC_DEV void tile_terms(const TileProblem& P, int dtype, uint64_t lo, uint64_t hi, uint32_t lane, const Each& each) {
    if (lo >= hi) return;                  /* a tile past the end of its problem */
    uint64_t rest = lo;
    uint32_t esz = dtype == DT_I8 ? 1u : 2u;
    if (WIDE && !P.sub && (dtype == DT_I8 || dtype == DT_I16 || dtype == DT_SPLIT16 || dtype == DT_SPLIT16M) && (((uintptr_t)P.scalars + lo * esz) & 15u) == 0) {
        uint32_t per = 16u / esz;
        uint64_t chunks = (hi - lo) / per;
        const Words16* src = (const Words16*)((const uint8_t*)P.scalars + lo * esz);
        for (uint64_t ch = lane; ch < chunks; ch += BLOCK) {
            Words16 x = src[ch];
            uint64_t i = lo + ch * per;
            if (esz == 2u) {
#pragma unroll
                for (int k = 0; k < 8; ++k) each(i + k, (int32_t)(int16_t)(x.w[k >> 1] >> (16 * (k & 1))));
            } else {
#pragma unroll
                for (int k = 0; k < 16; ++k) each(i + k, (int32_t)(int8_t)(x.w[k >> 2] >> (8 * (k & 3))));
            }
        }
        rest = lo + chunks * per;
    }
    for (uint64_t i = rest + lane; i < hi; i += BLOCK) each(i, tile_value(P, dtype, i));
}
template <int NBK, int LANES = 1024>            /* keys per problem = windows * buckets per window; lanes of a workgroup */
struct CountTile {
    static constexpr int BLOCK = LANES;
    static constexpr int PHASES = 3;
    static constexpr size_t LDS_BYTES = NBK * sizeof(uint32_t);
    const TileProblem* prob;
    int dtype, W, c;
    uint32_t n_wg;            /* tiles per problem */
    uint32_t* M;              /* problems * n_wg * NBK */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* hist = (uint32_t*)lds;
        uint32_t p = wg / n_wg, tl = wg % n_wg;
        const bool merged = dtype == DT_SPLIT16M;          /* all digits of a term share the one window */
        uint32_t nb = merged ? 0u : (uint32_t)NBK / (uint32_t)W;
        if (ph == 0) {
            for (uint32_t k = lane; k < (uint32_t)NBK; k += BLOCK) hist[k] = 0;
        } else if (ph == 1) {
            const TileProblem P = prob[p];
            uint64_t lo = (uint64_t)tl * P.tile, hi = lo + P.tile < P.n ? lo + P.tile : P.n;
            if ((NBK == 4096 && dtype == DT_FR) || (NBK == 2176 && dtype == DT_FR128)) {          /* full-width (or half-width) scalars in 8-bit windows: W digits per term */
                for (uint64_t i = lo + lane; i < hi; i += BLOCK) {
                    const uint32_t* v = ((const fr_plain*)P.scalars)[i].l;
                    uint32_t carry = 0;
                    for (int w = 0; w < W; ++w) {
                        int32_t d = fr_window_digit(v, w, c, carry);
                        if (d) atomic_add_u32(&hist[(uint32_t)w * nb + (uint32_t)(d < 0 ? -d : d) - 1u], 1u);
                    }
                }
                return;
            }
            tile_terms<BLOCK, NBK != 512>(P, dtype, lo, hi, lane, [&](uint64_t, int32_t v) {
                uint32_t mag = (uint32_t)(v < 0 ? -v : v), carry = 0;
                for (int w = 0; w < W; ++w) {
                    int32_t d = W == 1 ? (int32_t)mag : small_window_digit(mag, w, c, carry);
                    if (d) atomic_add_u32(&hist[(uint32_t)w * nb + (uint32_t)(d < 0 ? -d : d) - 1u], 1u);
                }
            });
        } else {
            uint32_t* row = M + (uint64_t)wg * NBK;
            for (uint32_t k = lane; k < (uint32_t)NBK; k += BLOCK) row[k] = hist[k];
        }
    }
};
struct TileColumnScan {       /* lane = (problem, key) */
    uint32_t nb, n_wg;
    uint32_t* M;
    uint32_t* cnt;            /* problems * nb */
    TC_DEV void operator()(uint32_t t) const {
        uint32_t p = t / nb, key = t % nb;
        uint32_t* col = M + (uint64_t)p * n_wg * nb + key;
        uint32_t off = 0, w = 0;
        /* sixteen loads in flight: taken one at a time, each waits for the one before (a lone flat commitment with
         * 256 tiles: 69 us that way) */
        for (; w + 16 <= n_wg; w += 16) {
            uint32_t v[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] = col[(uint64_t)(w + k) * nb];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                col[(uint64_t)(w + k) * nb] = off;
                off += v[k];
            }
        }
        for (; w < n_wg; ++w) {
            uint32_t v = col[(uint64_t)w * nb];
            col[(uint64_t)w * nb] = off;
            off += v;
        }
        cnt[t] = off;
    }
};
template <int NBK, int LANES = 1024>
struct ScatterTile {
    static constexpr int BLOCK = LANES;
    static constexpr int PHASES = 2;
    static constexpr size_t LDS_BYTES = NBK * sizeof(uint32_t);
    const TileProblem* prob;
    int dtype, W, c;
    uint32_t n_wg;
    const uint32_t* M;
    const uint32_t* start;    /* global bucket starts, problems * NBK (+1) */
    uint32_t* sorted;
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* cur = (uint32_t*)lds;
        uint32_t p = wg / n_wg, tl = wg % n_wg;
        const bool merged = dtype == DT_SPLIT16M;
        uint32_t nb = merged ? 0u : (uint32_t)NBK / (uint32_t)W;
        if (ph == 0) {
            const uint32_t* row = M + (uint64_t)wg * NBK;
            const uint32_t* st = start + (uint64_t)p * NBK;
            for (uint32_t k = lane; k < (uint32_t)NBK; k += BLOCK) cur[k] = st[k] + row[k];
        } else {
            const TileProblem P = prob[p];
            uint64_t lo = (uint64_t)tl * P.tile, hi = lo + P.tile < P.n ? lo + P.tile : P.n;
            if ((NBK == 4096 && dtype == DT_FR) || (NBK == 2176 && dtype == DT_FR128)) {
                for (uint64_t i = lo + lane; i < hi; i += BLOCK) {
                    const uint32_t* v = ((const fr_plain*)P.scalars)[i].l;
                    uint32_t carry = 0;
                    for (int w = 0; w < W; ++w) {
                        int32_t d = fr_window_digit(v, w, c, carry);
                        if (d) {
                            uint32_t pos = atomic_add_u32(&cur[(uint32_t)w * nb + (uint32_t)(d < 0 ? -d : d) - 1u], 1u);
                            sorted[pos] = (uint32_t)i | (d < 0 ? 0x80000000u : 0u);
                        }
                    }
                }
                return;
            }
            tile_terms<BLOCK, NBK != 512>(P, dtype, lo, hi, lane, [&](uint64_t i, int32_t v) {
                uint32_t mag = (uint32_t)(v < 0 ? -v : v), carry = 0;
                for (int w = 0; w < W; ++w) {
                    int32_t d = W == 1 ? (int32_t)mag : small_window_digit(mag, w, c, carry);
                    if (d) {
                        uint32_t pos = atomic_add_u32(&cur[(uint32_t)w * nb + (uint32_t)(d < 0 ? -d : d) - 1u], 1u);
                        bool negative = (d < 0) != (v < 0);
                        uint32_t idx = (uint32_t)i + (merged ? (uint32_t)w * P.shift : 0u);
                        sorted[pos] = idx | (negative ? 0x80000000u : 0u);
                    }
                }
            });
        }
    }
};

/* ---- counting sort of 16-bit magnitudes in two levels, tiles sorted in LDS ------------
 * ScatterTile<32768> sends every 4-byte entry to a memory line of its own: a tile's share of a bucket is a few
 * entries, no cache holds the 32768 open lines of every workgroup, and memory writes a whole sector per entry
 * (3.3 ms for the 3.1e8 entries of the LLaMA2-7B-shaped forward).  Sorting by the upper bits of the key
 * (magnitude - 1) first and by the lower `low` bits afterwards keeps the open lines few, but as long as every lane
 * sends its own 4-byte write each pass is bound by the L2's one request per channel and clock (1.3 ms).  So both
 * passes sort a tile of SORT_TILE entries in LDS first -- rank of every entry among those of its key from an LDS
 * atomic, prefix sums of the tile's histogram, entries placed in key order -- and write it out as runs: neighbouring
 * lanes write neighbouring words.  On the way from the first pass to the second an entry is one word: the index in
 * bits 0 .. 30 - low, above it the lower key bits, bit 31 the sign.  low = 7 (256 bins of 128 keys) for problems of
 * up to 2^24 terms, low = 6 (512 bins of 64 keys) up to 2^25. */
constexpr uint32_t SORT_KEY_BITS = 15;
constexpr uint32_t SORT_BINS_MAX = 512;      /* bins per problem (upper key bits) at low = 6 */
constexpr uint32_t SORT_KEYS_MAX = 128;      /* keys per bin (lower key bits) at low = 7 */
#if defined(TC_HOST_EMU)
constexpr uint32_t SORT_TILE = 64;           /* the CPU build of the tests meets several tiles per bin at its sizes */
#else
constexpr uint32_t SORT_TILE = 8192;         /* entries a workgroup sorts in LDS */
#endif
constexpr uint32_t SORT_NO_RANK = 0xFFFFu;
TC_HD uint32_t sort_pack(uint32_t i, uint32_t key, bool negative, uint32_t low) {
    return i | ((key & ((1u << low) - 1u)) << (31u - low)) | (negative ? 0x80000000u : 0u);
}
TC_HD uint32_t sort_low_key(uint32_t w, uint32_t low) { return (w >> (31u - low)) & ((1u << low) - 1u); }
TC_HD uint32_t sort_entry(uint32_t w, uint32_t low) { return w & (0x80000000u | ((1u << (31u - low)) - 1u)); }

/* largest b with off[b] <= j, off[0] = 0 non-decreasing, n a power of two */
TC_HD uint32_t sort_owner(const uint32_t* off, uint32_t n, uint32_t j) {
    uint32_t b = 0;
    for (uint32_t step = n >> 1; step; step >>= 1)
        if (off[b + step] <= j) b += step;
    return b;
}
/* off[k] = hist[0] + .. + hist[k - 1] for k <= n, by the first n lanes: every lane adds up its own prefix */
TC_DEV void sort_prefix(const uint32_t* hist, uint32_t n, uint32_t lane, uint32_t* off) {
    if (lane >= n) return;
    uint32_t at = 0;
    for (uint32_t k = 0; k < lane; ++k) at += hist[k];
    off[lane] = at;
    if (lane == n - 1) off[n] = at + hist[lane];
}
struct CountBins {             /* workgroup = (problem, tile): terms per bin */
    static constexpr int BLOCK = 512;
    static constexpr int PHASES = 3;
    static constexpr size_t LDS_BYTES = SORT_BINS_MAX * sizeof(uint32_t);
    static_assert(BLOCK >= (int)SORT_BINS_MAX, "a lane per bin");
    const TileProblem* prob;
    uint32_t n_wg, low;
    uint32_t* M;               /* problems * n_wg * bins per problem */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* hist = (uint32_t*)lds;
        uint32_t p = wg / n_wg, tl = wg % n_wg;
        const uint32_t nbins = 1u << (SORT_KEY_BITS - low);
        if (ph == 0) {
            if (lane < nbins) hist[lane] = 0;
        } else if (ph == 1) {
            const TileProblem P = prob[p];
            uint64_t lo = (uint64_t)tl * P.tile, hi = lo + P.tile < P.n ? lo + P.tile : P.n;
            tile_terms<BLOCK, true>(P, DT_I16, lo, hi, lane, [&](uint64_t, int32_t v) {
                uint32_t mag = (uint32_t)(v < 0 ? -v : v);
                if (mag) atomic_add_u32(&hist[(mag - 1u) >> low], 1u);
            });
        } else {
            if (lane < nbins) M[(uint64_t)wg * nbins + lane] = hist[lane];
        }
    }
};
struct ScatterBins {           /* the same workgroups (tiles of at most SORT_TILE terms): their entries, bin by bin */
    static constexpr int BLOCK = 512;
    static constexpr int PHASES = 5;
    /* histogram, its prefix sums (+ total), the tile's cursors; ranks; the tile in bin order */
    static constexpr size_t LDS_BYTES = (3 * SORT_BINS_MAX + 1) * sizeof(uint32_t) + SORT_TILE * sizeof(uint16_t) + SORT_TILE * sizeof(uint32_t);
    static_assert(BLOCK >= (int)SORT_BINS_MAX, "a lane per bin");
    const TileProblem* prob;
    uint32_t n_wg, low;
    const uint32_t* M;         /* after TileColumnScan: offset of the tile within its bin */
    const uint32_t* start;     /* bin starts, problems * bins per problem */
    uint32_t* packed;
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* hist = (uint32_t*)lds;
        uint32_t* off = hist + SORT_BINS_MAX;              /* bins + 1 */
        uint32_t* cur = off + SORT_BINS_MAX + 1;
        uint32_t* tile = cur + SORT_BINS_MAX;
        uint16_t* rank = (uint16_t*)(tile + SORT_TILE);
        uint32_t p = wg / n_wg, tl = wg % n_wg;
        const uint32_t nbins = 1u << (SORT_KEY_BITS - low);
        const TileProblem P = prob[p];
        uint64_t lo = (uint64_t)tl * P.tile, hi = lo + P.tile < P.n ? lo + P.tile : P.n;
        if (ph == 0) {
            if (lane < nbins) {
                hist[lane] = 0;
                cur[lane] = start[(uint64_t)p * nbins + lane] + M[(uint64_t)wg * nbins + lane];
            }
        } else if (ph == 1) {
            tile_terms<BLOCK, true>(P, DT_I16, lo, hi, lane, [&](uint64_t i, int32_t v) {
                uint32_t mag = (uint32_t)(v < 0 ? -v : v);
                rank[i - lo] = mag ? (uint16_t)atomic_add_u32(&hist[(mag - 1u) >> low], 1u) : (uint16_t)SORT_NO_RANK;
            });
        } else if (ph == 2) {
            sort_prefix(hist, nbins, lane, off);
        } else if (ph == 3) {
            tile_terms<BLOCK, true>(P, DT_I16, lo, hi, lane, [&](uint64_t i, int32_t v) {
                uint32_t mag = (uint32_t)(v < 0 ? -v : v);
                if (mag) tile[off[(mag - 1u) >> low] + rank[i - lo]] = sort_pack((uint32_t)i, mag - 1u, v < 0, low);
            });
        } else {
            uint32_t total = off[nbins];
            for (uint32_t j = lane; j < total; j += BLOCK) {
                uint32_t b = sort_owner(off, nbins, j);
                packed[cur[b] + (j - off[b])] = tile[j];
            }
        }
    }
};
/* Second level.  The stretch of a bin is cut into tiles of SORT_TILE entries; tile s of the launch is tile
 * s - tstart[b] of the bin b that owns it (tstart: prefix sums of the tiles per bin; owner[s] = b). */
struct SortTileOwners {        /* lane = bin */
    const uint32_t* tstart;
    uint32_t* owner;
    TC_DEV void operator()(uint32_t b) const {
        for (uint32_t s = tstart[b]; s < tstart[b + 1]; ++s) owner[s] = b;
    }
};
/* bin, first and last + 1 entry of tile s -> r[0..2]; a workgroup past the last tile gets an empty stretch of bin 0 */
TC_DEV void sort_tile_range(const uint32_t* start, const uint32_t* tstart, const uint32_t* owner, uint32_t bins, uint32_t s, uint32_t* r) {
    if (s >= tstart[bins]) {
        r[0] = r[1] = r[2] = 0;
        return;
    }
    uint32_t b = owner[s];
    uint32_t lo = start[b] + (s - tstart[b]) * SORT_TILE, end = start[b + 1];
    r[0] = b;
    r[1] = lo;
    r[2] = end - lo < SORT_TILE ? end : lo + SORT_TILE;
}
struct CountKeys {             /* workgroup = tile of the packed array: entries per key */
    static constexpr int BLOCK = 512;
    static constexpr int PHASES = 3;
    static constexpr size_t LDS_BYTES = (SORT_KEYS_MAX + 3) * sizeof(uint32_t);
    const uint32_t* packed;
    const uint32_t* start;     /* bin starts, bins + 1 */
    const uint32_t* tstart;    /* first tile of every bin, bins + 1 */
    const uint32_t* owner;
    uint32_t bins, low;
    uint32_t* T;               /* tiles * keys per bin */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* hist = (uint32_t*)lds;
        uint32_t* r = hist + SORT_KEYS_MAX;
        const uint32_t nkeys = 1u << low;
        if (ph == 0) {
            if (lane < nkeys) hist[lane] = 0;
            if (lane == SORT_KEYS_MAX) sort_tile_range(start, tstart, owner, bins, wg, r);
        } else if (ph == 1) {
            for (uint32_t i = r[1] + lane; i < r[2]; i += BLOCK) atomic_add_u32(&hist[sort_low_key(packed[i], low)], 1u);
        } else {
            if (lane < nkeys) T[(uint64_t)wg * nkeys + lane] = hist[lane];
        }
    }
};
struct KeyColumnScan {         /* lane = (bin, key): offsets of the bin's tiles within the bucket, bucket count */
    const uint32_t* tstart;
    uint32_t low;
    uint32_t* T;
    uint32_t* cnt;             /* bins * keys per bin */
    TC_DEV void operator()(uint32_t t) const {
        const uint32_t nkeys = 1u << low;
        uint32_t b = t >> low, key = t & (nkeys - 1u);
        uint32_t at = 0;
        for (uint32_t s = tstart[b]; s < tstart[b + 1]; ++s) {
            uint32_t v = T[(uint64_t)s * nkeys + key];
            T[(uint64_t)s * nkeys + key] = at;
            at += v;
        }
        cnt[t] = at;
    }
};
struct SortKeys {              /* the tiles of CountKeys: entries in bucket order, as ScatterTile writes them */
    static constexpr int BLOCK = 1024;
    static constexpr int PHASES = 5;
    static constexpr size_t LDS_BYTES = (3 * SORT_KEYS_MAX + 4) * sizeof(uint32_t) + SORT_TILE * sizeof(uint16_t) + SORT_TILE * sizeof(uint32_t);
    const uint32_t* packed;
    const uint32_t* start;     /* bin starts */
    const uint32_t* tstart;
    const uint32_t* owner;
    uint32_t bins, low;
    const uint32_t* T;         /* after KeyColumnScan */
    const uint32_t* bucket_start;      /* bins * keys per bin */
    uint32_t* sorted;          /* index | sign << 31 */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* hist = (uint32_t*)lds;
        uint32_t* off = hist + SORT_KEYS_MAX;              /* keys + 1 */
        uint32_t* cur = off + SORT_KEYS_MAX + 1;
        uint32_t* r = cur + SORT_KEYS_MAX;
        uint32_t* tile = r + 3;
        uint16_t* rank = (uint16_t*)(tile + SORT_TILE);
        const uint32_t nkeys = 1u << low;
        if (ph == 0) {
            if (lane < nkeys) hist[lane] = 0;
            if (lane == SORT_KEYS_MAX) sort_tile_range(start, tstart, owner, bins, wg, r);
        } else if (ph == 1) {
            if (lane < nkeys) cur[lane] = bucket_start[(uint64_t)r[0] * nkeys + lane] + T[(uint64_t)wg * nkeys + lane];
            for (uint32_t j = lane; r[1] + j < r[2]; j += BLOCK) rank[j] = (uint16_t)atomic_add_u32(&hist[sort_low_key(packed[r[1] + j], low)], 1u);
        } else if (ph == 2) {
            sort_prefix(hist, nkeys, lane, off);
        } else if (ph == 3) {
            for (uint32_t j = lane; r[1] + j < r[2]; j += BLOCK) {
                uint32_t w = packed[r[1] + j];
                tile[off[sort_low_key(w, low)] + rank[j]] = w;
            }
        } else {
            for (uint32_t j = lane; r[1] + j < r[2]; j += BLOCK) {
                uint32_t w = tile[j], key = sort_low_key(w, low);
                sorted[cur[key] + (j - off[key])] = sort_entry(w, low);
            }
        }
    }
};

/* ---- prefix sums over bucket counts (three lane-independent steps) ---------------- */
/* chunk = 256 consecutive buckets.  A: per-chunk totals of cnt and of ceil(cnt / L);
 * B: one lane turns the chunk totals into exclusive offsets; C: per-chunk serial prefix. */
constexpr uint32_t SCAN_CHUNK = 256;

struct ScanChunkTotals {
    const uint32_t* cnt;
    uint32_t n, L;
    uint32_t* tot_a;
    uint32_t* tot_b;
    uint32_t* tot_max;     /* per chunk: largest count */
    TC_DEV void operator()(uint32_t ch) const {
        uint32_t lo = ch * SCAN_CHUNK, hi = lo + SCAN_CHUNK < n ? lo + SCAN_CHUNK : n;
        uint32_t a = 0, b = 0, mx = 0;
        for (uint32_t i = lo; i < hi; ++i) {
            uint32_t v = cnt[i];
            a += v;
            b += (v + L - 1) / L;
            mx = v > mx ? v : mx;
        }
        tot_a[ch] = a;
        tot_b[ch] = b;
        tot_max[ch] = mx;
    }
};
struct ScanChunkOffsets {     /* one workgroup: every lane owns a slice of the chunk totals */
    static constexpr int BLOCK = 1024;
    static constexpr int PHASES = 3;
    static constexpr size_t LDS_BYTES = 3 * BLOCK * sizeof(uint32_t);
    uint32_t nchunks;
    uint32_t* tot_a;
    uint32_t* tot_b;
    uint32_t* tot_max;     /* in: per-chunk maxima; out: tot_max[nchunks] = overall maximum */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t, uint8_t* lds) const {
        uint32_t* sa = (uint32_t*)lds;
        uint32_t* sb = sa + BLOCK;
        uint32_t* sm = sb + BLOCK;
        uint32_t per = (nchunks + BLOCK - 1) / BLOCK;
        uint32_t lo = lane * per < nchunks ? lane * per : nchunks;
        uint32_t hi = lo + per < nchunks ? lo + per : nchunks;
        if (ph == 0) {
            uint32_t a = 0, b = 0, mx = 0;
            for (uint32_t i = lo; i < hi; ++i) {
                a += tot_a[i];
                b += tot_b[i];
                mx = tot_max[i] > mx ? tot_max[i] : mx;
            }
            sa[lane] = a; sb[lane] = b; sm[lane] = mx;
        } else if (ph == 1) {
            if (lane == 0) {
                uint32_t a = 0, b = 0, mx = 0;
                for (uint32_t i = 0; i < (uint32_t)BLOCK; ++i) {
                    uint32_t va = sa[i], vb = sb[i];
                    sa[i] = a; sb[i] = b;
                    a += va; b += vb;
                    mx = sm[i] > mx ? sm[i] : mx;
                }
                tot_a[nchunks] = a;
                tot_b[nchunks] = b;
                tot_max[nchunks] = mx;
            }
        } else {
            uint32_t a = sa[lane], b = sb[lane];
            for (uint32_t i = lo; i < hi; ++i) {
                uint32_t va = tot_a[i], vb = tot_b[i];
                tot_a[i] = a;
                tot_b[i] = b;
                a += va;
                b += vb;
            }
        }
    }
};
struct ScanWrite {
    const uint32_t* cnt;
    uint32_t n, L;
    const uint32_t* tot_a;
    const uint32_t* tot_b;
    uint32_t nchunks;
    uint32_t* start;     /* n + 1 */
    uint32_t* lstart;    /* n + 1 */
    uint32_t* zero_me;   /* optional array of n counters to clear (scatter cursors) */
    TC_DEV void operator()(uint32_t ch) const {
        uint32_t lo = ch * SCAN_CHUNK, hi = lo + SCAN_CHUNK < n ? lo + SCAN_CHUNK : n;
        uint32_t a = tot_a[ch], b = tot_b[ch];
        for (uint32_t i = lo; i < hi; ++i) {
            uint32_t v = cnt[i];
            start[i] = a;
            lstart[i] = b;
            a += v;
            b += (v + L - 1) / L;
            if (zero_me) zero_me[i] = 0;
        }
        if (ch == nchunks - 1) {
            start[n] = tot_a[nchunks];
            lstart[n] = tot_b[nchunks];
        }
    }
};
/* The same prefix sums in one launch when there are few buckets (n <= MAX_N): one workgroup, every lane owns
 * ceil(n / BLOCK) consecutive buckets.  The three launches above take about 100 us for 32768 buckets, most of it the
 * serial loops of their few lanes; a flat commitment of 2^21 terms runs the scan once per pass. */
struct ScanSmall {
    static constexpr int BLOCK = 1024;
    static constexpr int GROUP = 32;           /* lanes per group of the two-level scan over the lanes' sums */
    static constexpr int PHASES = 5;
    static constexpr size_t LDS_BYTES = (3 * BLOCK + 2 * (BLOCK / GROUP)) * sizeof(uint32_t);
    static constexpr uint32_t MAX_N = 65536;
    const uint32_t* cnt;
    uint32_t n, L;
    uint32_t* start;       /* n + 1 */
    uint32_t* lstart;      /* n + 1 */
    uint32_t* zero_me;     /* optional */
    uint32_t* total_a;     /* one value each: sum of cnt, sum of ceil(cnt / L), largest cnt */
    uint32_t* total_b;
    uint32_t* total_max;
    /* ceil(v / L) without a division per bucket: L <= 64, and floor(x / L) = (x * ceil(2^32 / L)) >> 32 for x < 2^26 */
    TC_DEV uint32_t lanes_for(uint32_t v, uint32_t magic) const {
        uint32_t x = v + L - 1;
        return x < (1u << 26) ? (uint32_t)(((uint64_t)x * magic) >> 32) : x / L;
    }
    struct Quad { uint32_t v[4]; };
    TC_DEV void phase(int ph, uint32_t lane, uint32_t, uint8_t* lds) const {
        uint32_t* sa = (uint32_t*)lds;
        uint32_t* sb = sa + BLOCK;
        uint32_t* sm = sb + BLOCK;
        uint32_t* ga = sm + BLOCK;             /* per group of lanes */
        uint32_t* gb = ga + BLOCK / GROUP;
        uint32_t per = (n + BLOCK - 1) / BLOCK;
        uint32_t lo = lane * per < n ? lane * per : n;
        uint32_t hi = lo + per < n ? lo + per : n;
        uint32_t magic = L > 1 ? (uint32_t)(((1ull << 32) + L - 1) / L) : 0u;         /* L = 1: the quotient is the count itself */
        /* a lane's buckets as 16-byte pieces when they are whole pieces (32768 buckets: 32 per lane) */
        bool quads = (per & 3u) == 0 && hi - lo == per && (((uintptr_t)cnt | (uintptr_t)start | (uintptr_t)lstart) & 15u) == 0;
        if (ph == 0) {                         /* every lane: sums over its own buckets */
            uint32_t a = 0, b = 0, mx = 0;
            if (quads) {
                const Quad* c4 = (const Quad*)(cnt + lo);
                for (uint32_t i = 0; i < per / 4; ++i) {
                    Quad q = c4[i];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        uint32_t v = q.v[k];
                        a += v;
                        b += L > 1 ? lanes_for(v, magic) : v;
                        mx = v > mx ? v : mx;
                    }
                }
            } else {
                for (uint32_t i = lo; i < hi; ++i) {
                    uint32_t v = cnt[i];
                    a += v;
                    b += L > 1 ? lanes_for(v, magic) : v;
                    mx = v > mx ? v : mx;
                }
            }
            sa[lane] = a; sb[lane] = b; sm[lane] = mx;
        } else if (ph == 1) {                  /* one lane per group: exclusive prefix inside the group, the group's totals */
            if (lane < (uint32_t)(BLOCK / GROUP)) {
                uint32_t a = 0, b = 0, mx = 0;
                for (uint32_t i = lane * GROUP; i < (lane + 1) * GROUP; ++i) {
                    uint32_t va = sa[i], vb = sb[i];
                    sa[i] = a; sb[i] = b;
                    a += va; b += vb;
                    mx = sm[i] > mx ? sm[i] : mx;
                }
                ga[lane] = a; gb[lane] = b; sm[lane * GROUP] = mx;
            }
        } else if (ph == 2) {                  /* one lane: exclusive prefix over the groups, the grand totals */
            if (lane == 0) {
                uint32_t a = 0, b = 0, mx = 0;
                for (uint32_t g = 0; g < (uint32_t)(BLOCK / GROUP); ++g) {
                    uint32_t va = ga[g], vb = gb[g];
                    ga[g] = a; gb[g] = b;
                    a += va; b += vb;
                    mx = sm[g * GROUP] > mx ? sm[g * GROUP] : mx;
                }
                *total_a = a;
                *total_b = b;
                *total_max = mx;
                start[n] = a;
                lstart[n] = b;
            }
        } else if (ph == 3) {
            sa[lane] += ga[lane / GROUP];
            sb[lane] += gb[lane / GROUP];
        } else {
            uint32_t a = sa[lane], b = sb[lane];
            if (quads && !zero_me) {
                const Quad* c4 = (const Quad*)(cnt + lo);
                Quad* s4 = (Quad*)(start + lo);
                Quad* l4 = (Quad*)(lstart + lo);
                for (uint32_t i = 0; i < per / 4; ++i) {
                    Quad q = c4[i], qs, ql;
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        uint32_t v = q.v[k];
                        qs.v[k] = a;
                        ql.v[k] = b;
                        a += v;
                        b += L > 1 ? lanes_for(v, magic) : v;
                    }
                    s4[i] = qs;
                    l4[i] = ql;
                }
            } else {
                for (uint32_t i = lo; i < hi; ++i) {
                    uint32_t v = cnt[i];
                    start[i] = a;
                    lstart[i] = b;
                    a += v;
                    b += L > 1 ? lanes_for(v, magic) : v;
                    if (zero_me) zero_me[i] = 0;
                }
            }
        }
    }
};
/* cnt[i] = prefix[i + 1] - prefix[i] */
struct DiffCounts {
    const uint32_t* prefix;
    uint32_t* cnt;
    TC_DEV void operator()(uint32_t t) const { cnt[t] = prefix[t + 1] - prefix[t]; }
};

/* largest b in [0, n) with prefix[b] <= t, for a non-decreasing prefix with prefix[n] > t */
TC_HD uint32_t find_segment(const uint32_t* prefix, uint32_t n, uint32_t t) {
    uint32_t lo = 0, hi = n;       /* invariant: prefix[lo] <= t < prefix[hi] */
    while (hi - lo > 1) {
        uint32_t mid = lo + ((hi - lo) >> 1);
        if (prefix[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

/* ---- MSM: balanced segmented sums per bucket -------------------------------------- */
/* The accumulator lives in the 28-bit-limb form of the field (carry-free products and additions, expanded in place:
 * the loop is 3542 multiply-adds and little else); points enter by a re-cut of their limbs, the sum leaves through
 * one full reduction per coordinate.  The chord rule runs without its case distinctions.  When its denominator may
 * be zero in the field (equal or opposite points; told from its two lowest limbs, which practically no other value
 * passes) the lane gives its sub-run up and enters it in a list, and a second launch (AccAffineRedo) sums the
 * listed sub-runs with the routine that settles every case. */
/* acc += (x2, y2), both finite; false (acc unusable) when the sum may be a doubling or the identity.
 * |P| <= 317 p in the first addition after acc was a re-cut affine point (coordinates 2^8 times larger than a
 * reduced value), <= 43 p in the second, <= 5 p from then on. */
TC_HD bool xyzz28_madd_regular(g1_xyzz28& a, const fp28& x2, const fp28& y2) {
    fp28 P = fp28_sub(fp28_mul_inline(x2, a.ZZ), a.X);
    if (fp28_maybe_zero(P, 512u)) return false;
    fp28 R = fp28_sub(fp28_mul_inline(y2, a.ZZZ), a.Y);
    fp28 PP = fp28_sqr_inline(P);
    fp28 PPP = fp28_mul_inline(P, PP);
    fp28 Q = fp28_mul_inline(a.X, PP);
    fp28 X3 = fp28_carry(fp28_sub(fp28_sub(fp28_sub(fp28_sqr_inline(R), PPP), Q), Q));
    a.Y = fp28_mul_sub_inline(R, fp28_sub(Q, X3), a.Y, PPP);          /* limbs below 2^29 against 2^28, twice */
    a.ZZ = fp28_mul_inline(a.ZZ, PP);
    a.ZZZ = fp28_mul_inline(a.ZZZ, PPP);
    a.X = X3;
    return true;
}
/* Tables of the accumulation.  A table of 96-byte points at a stride of 96 bytes puts every second point across two
 * of the 128-byte lines in which the second-level cache fetches: 192 bytes per point gathered at a random index.
 * The SRS therefore keeps a copy of its first table at a stride of 128 bytes for the launches that gather from it;
 * other tables (suffix tables, row commitments used as bases) stay at 96.  A table pointer carries its kind in
 * bit 0 (tables start on 16-byte boundaries).
 * The 128 bytes have room for the point as the accumulation wants it: words 0..13 the 28-bit limbs of x, 14..27 those
 * of y (fp28_from_fp), so that a lane neither re-cuts the 32-bit limbs of every point it adds (56 instructions) nor
 * tests 24 words for the identity, which has -1 as the top limb of y (that limb of a point is below 2^28). */
constexpr uint32_t PADDED_STRIDE = 128;
struct PaddedPoint {
    fp28 x, y;
    uint32_t unused[4];
};
static_assert(sizeof(PaddedPoint) == PADDED_STRIDE, "one point per 128-byte line");
TC_HD const g1_affine* tag_padded(const void* table) { return (const g1_affine*)((uintptr_t)table | 1u); }
TC_HD bool table_is_padded(const g1_affine* tagged) { return ((uintptr_t)tagged & 1u) != 0; }
TC_HD const PaddedPoint* padded_point(const g1_affine* tagged, uint32_t i) {
    return (const PaddedPoint*)(((uintptr_t)tagged & ~(uintptr_t)15u) + (uint64_t)i * PADDED_STRIDE);
}
/* limbs of x and y from seven 16-byte loads */
TC_HD void padded_load(const PaddedPoint* q, fp28& x, fp28& y) {
    Words16 c[7];
#pragma unroll
    for (int k = 0; k < 7; ++k) c[k] = ((const Words16*)q)[k];
#pragma unroll
    for (int j = 0; j < 14; ++j) {
        x.l[j] = (int32_t)c[j >> 2].w[j & 3];
        y.l[j] = (int32_t)c[(14 + j) >> 2].w[(14 + j) & 3];
    }
}
/* point i of either kind of table in the 32-bit form (the kernels off the fast path) */
TC_HD g1_affine table_point(const g1_affine* tagged, uint32_t i) {
    if (table_is_padded(tagged)) {
        fp28 x, y;
        padded_load(padded_point(tagged, i), x, y);
        if (y.l[13] < 0) return affine_identity();
        g1_affine p;
        p.x = fp28_recut_to_fp(x);
        p.y = fp28_recut_to_fp(y);
        return p;
    }
    return tagged[i];
}
struct PadPoints {            /* out: the points of `in`, one per 128 bytes, in 28-bit limbs */
    const g1_affine* in;
    uint8_t* out;
    TC_DEV void operator()(uint32_t t) const {
        g1_affine p = in[t];
        PaddedPoint v;
        v.x = fp28_from_fp(p.x);
        v.y = fp28_from_fp(p.y);
        if (affine_is_identity(p)) v.y.l[13] = -1;
#pragma unroll
        for (int k = 0; k < 4; ++k) v.unused[k] = 0;
        *(PaddedPoint*)(out + (uint64_t)t * PADDED_STRIDE) = v;
    }
};

/* Lane t owns sub-run `t - lstart[b]` of bucket b: at most L entries, all of one bucket.
 * Output slot t, so the partial sums of bucket b are the slots lstart[b] .. lstart[b+1].
 * The k = ceil(c / L) sub-runs of a bucket with c entries are equally long (to within one entry), not L, L, .., rest:
 * the lanes of a wave run for as long as the longest of their sub-runs, and neighbouring lanes share a bucket or have
 * buckets of similar loads. */
TC_HD void subrun_bounds(const uint32_t* start, const uint32_t* lstart, uint32_t b, uint32_t t, uint32_t& begin, uint32_t& end) {
    uint32_t s0 = start[b], c = start[b + 1] - s0;
    uint32_t l0 = lstart[b], k = lstart[b + 1] - l0, j = t - l0;
    uint32_t low = c / k, more = c - low * k;          /* the first `more` sub-runs hold one entry more than the others */
    begin = s0 + j * low + (j < more ? j : more);
    end = begin + low + (j < more ? 1u : 0u);
}
enum { TABLES_PLAIN = 0, TABLES_PADDED = 1, TABLES_MIXED = 2 };
/* What the launch gathers from.  Only the kernel for padded tables alone stays within the 168 registers of three waves
 * per SIMD (162); the other two spill some forty registers, which costs the full-width problems at the end of a batch
 * of openings about 3 % (4.0 -> 4.1 ms of 58). */
template <int TABLES>
struct AccAffine {
    const g1_affine* const* tables;   /* SRS table of problem p; bucket b belongs to problem b / nbk_pp */
    uint32_t nbk_pp;
    const uint32_t* sorted;
    const uint32_t* start;
    const uint32_t* lstart;
    uint32_t nbk, L;
    g1_xyzz* out;
    uint32_t* redo_count;             /* zero before the launch */
    uint32_t* redo_list;              /* room for every lane */
    const uint32_t* perm;             /* lane -> sub-run (lanes ordered by the length of their sub-runs), or null */
    TC_DEV void operator()(uint32_t lane) const {
        if (lane >= lstart[nbk]) return;
        uint32_t t = perm ? perm[lane] : lane;
        uint32_t b = find_segment(lstart, nbk, t);
        uint32_t begin, end;
        subrun_bounds(start, lstart, b, t, begin, end);
        const g1_affine* pts = tables[b / nbk_pp];                /* tagged with its stride */
        if (end - begin == 1) {                                   /* a lone entry: no arithmetic */
            uint32_t e = sorted[begin];
            g1_affine p = TABLES == TABLES_PLAIN ? pts[e & 0x7FFFFFFFu] : table_point(pts, e & 0x7FFFFFFFu);
            if (e >> 31) p.y = fp_neg(p.y);
            out[t] = xyzz_from_affine(p);
            return;
        }
        g1_xyzz28 acc;
        bool have = false;                                        /* acc holds a point (the sum so far is not the identity) */
        /* the indices come four at a time (the list starts on a 16-byte boundary and its allocation ends on one): an
         * addition lasts long enough for the other waves to push a line out of the caches, and a lane that fetches
         * its indices one by one pulls every line of its run in again and again */
        Words16 four = {{0u, 0u, 0u, 0u}};
        uint32_t held = 0xFFFFFFFFu;                              /* which group of four `four` holds */
        for (uint32_t i = begin; i < end; ++i) {
            if ((i >> 2) != held) {
                held = i >> 2;
                four = ((const Words16*)sorted)[held];
            }
            uint32_t j = i & 3u;
            uint32_t e = j == 0u ? four.w[0] : j == 1u ? four.w[1] : j == 2u ? four.w[2] : four.w[3];
            fp28 x2, y2;
            if (TABLES == TABLES_PADDED || (TABLES == TABLES_MIXED && table_is_padded(pts))) {
                padded_load(padded_point(pts, e & 0x7FFFFFFFu), x2, y2);
                if (y2.l[13] < 0) continue;
            } else {
                g1_affine p = pts[e & 0x7FFFFFFFu];
                if (affine_is_identity(p)) continue;
                x2 = fp28_from_fp(p.x);
                y2 = fp28_from_fp(p.y);
            }
            if (e >> 31) y2 = fp28_sub(fp28{}, y2);
            if (!have) {
                acc.X = x2;
                acc.Y = y2;
                acc.ZZ = fp28_one();
                acc.ZZZ = fp28_one();
                have = true;
                continue;
            }
            if (!xyzz28_madd_regular(acc, x2, y2)) {
                redo_list[atomic_add_u32(redo_count, 1u)] = t;
                return;
            }
        }
        g1_xyzz r;
        if (!have) {
            r = xyzz_identity();
        } else {
            r.X = fp28_to_fp_outlined(acc.X); r.Y = fp28_to_fp_outlined(acc.Y);
            r.ZZ = fp28_to_fp_outlined(acc.ZZ); r.ZZZ = fp28_to_fp_outlined(acc.ZZZ);
        }
        out[t] = r;
    }
};
/* ---- lanes of the accumulation ordered by the length of their sub-runs ---------------------------------------
 * The lanes of a wave run for as long as the longest of their sub-runs.  Where loads differ from bucket to bucket
 * (the rows of an opening: 30 to 170 entries per bucket side by side) lanes in bucket order leave a fifth of a wave's
 * lane-time idle; handed out in the order of their lengths, longest first, the sub-runs of a wave are equally long.
 * perm[lane] = sub-run; its output slot stays the sub-run's own, so nothing after the accumulation changes.
 * SubrunHist: one lane per bucket (k sub-runs of a bucket with c entries: c mod k of length c / k + 1, the others of
 * length c / k).  SubrunBinStarts: one lane.  SubrunOrder: one lane per bucket again (no search for the bucket of a
 * sub-run; the sub-runs of a bucket that has more than 64 of them -- one that holds most of a tensor has a million --
 * are placed by its whole workgroup); positions inside a bin are handed out by atomics, so the order inside a bin varies from run to
 * run -- the sums do not.  The passes over the partial sums
 * are ordered the same way; lstart = null stands for their last one, a lane per bucket over all that it holds. */
constexpr uint32_t SUBRUN_BINS = 65;          /* lengths 0 .. 63, and 64 or more */
TC_HD uint32_t subrun_bin(uint32_t len) { return len < SUBRUN_BINS - 1u ? len : SUBRUN_BINS - 1u; }
struct SubrunHist {
    static constexpr int BLOCK = 256;
    static constexpr int PHASES = 3;
    static constexpr size_t LDS_BYTES = SUBRUN_BINS * sizeof(uint32_t);
    const uint32_t* start;
    const uint32_t* lstart;
    uint32_t nbk;
    uint32_t* hist;              /* SUBRUN_BINS counters, zero before the launch */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* h = (uint32_t*)lds;
        if (ph == 0) {
            if (lane < SUBRUN_BINS) h[lane] = 0;
        } else if (ph == 1) {
            uint32_t b = wg * (uint32_t)BLOCK + lane;
            if (b >= nbk) return;
            uint32_t c = start[b + 1] - start[b];
            if (!lstart) {                   /* one lane per bucket, whatever it holds */
                atomic_add_u32(&h[subrun_bin(c)], 1u);
                return;
            }
            uint32_t k = lstart[b + 1] - lstart[b];
            if (!k) return;
            uint32_t base = c / k, more = c % k;
            if (more) atomic_add_u32(&h[subrun_bin(base + 1u)], more);
            atomic_add_u32(&h[subrun_bin(base)], k - more);
        } else if (lane < SUBRUN_BINS && h[lane]) {
            atomic_add_u32(&hist[lane], h[lane]);
        }
    }
};
struct SubrunBinStarts {         /* longest first */
    const uint32_t* hist;
    uint32_t* binstart;
    uint32_t* cursor;
    TC_DEV void operator()(uint32_t) const {
        uint32_t off = 0;
        for (uint32_t i = SUBRUN_BINS; i-- > 0;) {
            binstart[i] = off;
            cursor[i] = 0;
            off += hist[i];
        }
    }
};
struct SubrunOrder {             /* one lane per bucket, which places its sub-runs one after the other */
    static constexpr int BLOCK = 256;
    static constexpr int PHASES = 4;
    static constexpr size_t LDS_BYTES = (2 * SUBRUN_BINS + 1 + BLOCK) * sizeof(uint32_t);
    static constexpr uint32_t OWN_MAX = 64;      /* a bucket with more sub-runs than this is placed by the whole workgroup */
    const uint32_t* start;
    const uint32_t* lstart;
    uint32_t nbk;
    const uint32_t* binstart;
    uint32_t* cursor;            /* zero before the launch */
    uint32_t* perm;
    /* sub-runs of bucket b: its first slot, how many, and the entries that they share */
    TC_DEV void bucket(uint32_t b, uint32_t& slot0, uint32_t& k, uint32_t& c) const {
        c = start[b + 1] - start[b];
        if (!lstart) { slot0 = b; k = 1u; return; }
        slot0 = lstart[b];
        k = lstart[b + 1] - slot0;
    }
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t* cnt = (uint32_t*)lds;
        uint32_t* base = cnt + SUBRUN_BINS;
        uint32_t* n_big = base + SUBRUN_BINS;     /* buckets of this workgroup with more than OWN_MAX sub-runs ... */
        uint32_t* big = n_big + 1;                /* ... and which (a bucket that holds most of a tensor has a million) */
        uint32_t b = wg * (uint32_t)BLOCK + lane;
        if (ph == 0) {
            if (lane < SUBRUN_BINS) cnt[lane] = 0;
            if (lane == 0) *n_big = 0;
        } else if (ph == 1) {
            if (b >= nbk) return;
            uint32_t slot0, k, c;
            bucket(b, slot0, k, c);
            if (!k) return;
            uint32_t low = c / k, more = c % k;
            if (more) atomic_add_u32(&cnt[subrun_bin(low + 1u)], more);
            atomic_add_u32(&cnt[subrun_bin(low)], k - more);
            if (k > OWN_MAX) big[atomic_add_u32(n_big, 1u)] = b;
        } else if (ph == 2) {
            if (lane < SUBRUN_BINS) {
                base[lane] = cnt[lane] ? binstart[lane] + atomic_add_u32(&cursor[lane], cnt[lane]) : 0u;
                cnt[lane] = 0;
            }
        } else {
            uint32_t slot0, k, c;
            if (b < nbk) {
                bucket(b, slot0, k, c);
                if (k && k <= OWN_MAX) {
                    uint32_t low = lstart ? c / k : c, more = lstart ? c - low * k : 0u;
                    for (uint32_t j = 0; j < k; ++j) {
                        uint32_t bin = subrun_bin(low + (j < more ? 1u : 0u));
                        perm[base[bin] + atomic_add_u32(&cnt[bin], 1u)] = slot0 + j;
                    }
                }
            }
            for (uint32_t q = 0; q < *n_big; ++q) {
                bucket(big[q], slot0, k, c);
                uint32_t low = c / k, more = c - low * k;
                for (uint32_t j = lane; j < k; j += (uint32_t)BLOCK) {
                    uint32_t bin = subrun_bin(low + (j < more ? 1u : 0u));
                    perm[base[bin] + atomic_add_u32(&cnt[bin], 1u)] = slot0 + j;
                }
            }
        }
    }
};

/* the sub-runs that AccAffine gave up, summed with every case of the group law */
struct AccAffineRedo {
    const g1_affine* const* tables;
    uint32_t nbk_pp;
    const uint32_t* sorted;
    const uint32_t* start;
    const uint32_t* lstart;
    uint32_t nbk, L;
    g1_xyzz* out;
    const uint32_t* redo_count;
    const uint32_t* redo_list;
    uint32_t lanes;
    TC_DEV void operator()(uint32_t lane) const {
        for (uint32_t k = lane; k < *redo_count; k += lanes) {
            uint32_t t = redo_list[k];
            uint32_t b = find_segment(lstart, nbk, t);
            uint32_t begin, end;
            subrun_bounds(start, lstart, b, t, begin, end);
            const g1_affine* pts = tables[b / nbk_pp];
            xyzz_acc acc = acc_identity();
            for (uint32_t i = begin; i < end; ++i) {
                uint32_t e = sorted[i];
                acc_madd(acc, table_point(pts, e & 0x7FFFFFFFu), (e >> 31) != 0);
            }
            out[t] = acc_result(acc);
        }
    }
};
struct AccXyzz {
    const g1_xyzz* in;
    const uint32_t* start;     /* slots of bucket b in `in`: start[b] .. start[b+1] */
    const uint32_t* lstart;
    uint32_t nbk, L;
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t t) const {
        if (t >= lstart[nbk]) return;
        uint32_t b = find_segment(lstart, nbk, t);
        uint32_t begin = start[b] + (t - lstart[b]) * L;
        uint32_t end = begin + L < start[b + 1] ? begin + L : start[b + 1];
        if (end - begin == 1) { out[t] = in[begin]; return; }
        xyzz_acc acc = acc_from(in[begin]);
        for (uint32_t i = begin + 1; i < end; ++i) acc_add(acc, acc_from(in[i]));
        out[t] = acc_result(acc);
    }
};
/* The same passes for launches that fill the chip: the general addition expanded in place in the 28-bit form, no
 * call and no case distinction in the loop (as in AccAffine); a lane whose sum meets equal or opposite points gives
 * it up and enters it in a list that AccXyzzRedo works off with the routine that settles every case.  `final` = one
 * lane per bucket over all its partial sums (the last pass). */
struct AccXyzzFast {
    const g1_xyzz* in;
    const uint32_t* start;
    const uint32_t* lstart;
    uint32_t nbk, L;
    g1_xyzz* out;
    uint32_t* redo_count;
    uint32_t* redo_list;
    bool final;
    const uint32_t* perm;          /* lane -> slot, ordered by the number of sums behind the slot, or null */
    TC_DEV void operator()(uint32_t lane) const {
        uint32_t begin, end;
        if (lane >= (final ? nbk : lstart[nbk])) return;
        uint32_t t = perm ? perm[lane] : lane;
        if (final) {
            begin = start[t];
            end = start[t + 1];
        } else {
            uint32_t b = find_segment(lstart, nbk, t);
            subrun_bounds(start, lstart, b, t, begin, end);
        }
        if (end - begin <= 1) {
            out[t] = begin < end ? in[begin] : xyzz_identity();
            return;
        }
        g1_xyzz28 acc;
        bool have = false;
        for (uint32_t i = begin; i < end; ++i) {
            g1_xyzz p = in[i];
            if (xyzz_is_identity(p)) continue;
            g1_xyzz28 q = xyzz28_from(p);
            if (!have) {
                acc = q;
                have = true;
                continue;
            }
            if (!acc_add_regular_expanded(acc, q)) {
                redo_list[atomic_add_u32(redo_count, 1u)] = t;
                return;
            }
        }
        g1_xyzz r;
        if (!have) {
            r = xyzz_identity();
        } else {
            r.X = fp28_to_fp_outlined(acc.X); r.Y = fp28_to_fp_outlined(acc.Y);
            r.ZZ = fp28_to_fp_outlined(acc.ZZ); r.ZZZ = fp28_to_fp_outlined(acc.ZZZ);
        }
        out[t] = r;
    }
};
struct AccXyzzRedo {
    const g1_xyzz* in;
    const uint32_t* start;
    const uint32_t* lstart;
    uint32_t nbk, L;
    g1_xyzz* out;
    const uint32_t* redo_count;
    const uint32_t* redo_list;
    bool final;
    uint32_t lanes;
    TC_DEV void operator()(uint32_t lane) const {
        for (uint32_t k = lane; k < *redo_count; k += lanes) {
            uint32_t t = redo_list[k], begin, end;
            if (final) {
                begin = start[t];
                end = start[t + 1];
            } else {
                uint32_t b = find_segment(lstart, nbk, t);
                subrun_bounds(start, lstart, b, t, begin, end);
            }
            xyzz_acc acc = acc_from(in[begin]);
            for (uint32_t i = begin + 1; i < end; ++i) acc_add(acc, acc_from(in[i]));
            out[t] = acc_result(acc);
        }
    }
};
/* last pass: one lane per bucket sums whatever partials remain (bounded by the pass plan) */
struct AccFinal {
    const g1_xyzz* in;
    const uint32_t* start;
    g1_xyzz* bucket;
    TC_DEV void operator()(uint32_t b) const {
        uint32_t begin = start[b], end = start[b + 1];
        if (end - begin <= 1) { bucket[b] = begin < end ? in[begin] : xyzz_identity(); return; }
        xyzz_acc acc = acc_from(in[begin]);
        for (uint32_t i = begin + 1; i < end; ++i) acc_add(acc, acc_from(in[i]));
        bucket[b] = acc_result(acc);
    }
};

/* ---- sums of few points, where depth is the cost ------------------------------------------ */
/* One workgroup of four waves adds up to 256 XYZZ points pairwise, and the four waves share every addition:
 * its fourteen products fall into four levels of independent ones (U1 U2 S1 S2 | PP RR ZZa.ZZb ZZZa.ZZZb |
 * PPP Q ZZ' | T1 T2 ZZZ'), and a wave alone on its SIMD issues products no faster one after the other than four
 * waves do side by side, so an addition costs four product latencies instead of fourteen.  Points and
 * intermediates live in LDS, field by field (lanes of a wave touch consecutive 16-byte pieces); a barrier
 * separates the levels.  Reads of the operands happen in the first two levels, writes of the result (into the
 * slot of the first operand) in the last three, and only when the addition is a regular one; an identity
 * operand, opposite points and equal points are settled by wave 0 in the last level.
 *
 * `Src` says what is summed: count(wg) <= 256 slots, load(wg, i) the point of slot i, store(wg, sum). */
struct Quad16 { uint32_t v[4]; };
template <class Src>
struct CoopReduce {
    static constexpr int BLOCK = 256;
    static constexpr int NP = 256;
    enum { PX, PY, PZZ, PZZZ, NPF };
    enum { TU1, TU2, TS1, TS2, TPP, TRR, TZA, TZB, TPPP, TQ, NT };
    static constexpr int TP = 64;                                             /* pairs in flight: one per lane of a wave */
    static constexpr size_t TEMP_BASE = (size_t)NPF * 3 * NP;                 /* in 16-byte pieces */
    static constexpr size_t FLAG_BASE = (TEMP_BASE + (size_t)NT * 3 * TP) * 16;   /* in bytes */
    static constexpr size_t LDS_BYTES = FLAG_BASE + 3 * TP * 4;
    static constexpr int PHASES = 1 + 9 * 5 + 1;     /* load; the 128 pairs of the first level in two passes, seven more levels; store */
    Src src;

    TC_DEV static fp_t ldq(const uint8_t* lds, size_t base, int f, uint32_t n, uint32_t i) {
        const Quad16* q = (const Quad16*)lds + base;
        fp_t r;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            Quad16 t = q[(size_t)(f * 3 + k) * n + i];
            r.l[4 * k] = t.v[0]; r.l[4 * k + 1] = t.v[1]; r.l[4 * k + 2] = t.v[2]; r.l[4 * k + 3] = t.v[3];
        }
        return r;
    }
    TC_DEV static void stq(uint8_t* lds, size_t base, int f, uint32_t n, uint32_t i, const fp_t& x) {
        Quad16* q = (Quad16*)lds + base;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            Quad16 t;
            t.v[0] = x.l[4 * k]; t.v[1] = x.l[4 * k + 1]; t.v[2] = x.l[4 * k + 2]; t.v[3] = x.l[4 * k + 3];
            q[(size_t)(f * 3 + k) * n + i] = t;
        }
    }
    TC_DEV static fp_t pt(const uint8_t* lds, int f, uint32_t slot) { return ldq(lds, 0, f, NP, slot); }
    TC_DEV static void pt_set(uint8_t* lds, int f, uint32_t slot, const fp_t& x) { stq(lds, 0, f, NP, slot, x); }
    TC_DEV static fp_t tmp(const uint8_t* lds, int f, uint32_t t) { return ldq(lds, TEMP_BASE, f, TP, t); }
    TC_DEV static void tmp_set(uint8_t* lds, int f, uint32_t t, const fp_t& x) { stq(lds, TEMP_BASE, f, TP, t, x); }
    TC_DEV static g1_xyzz point(const uint8_t* lds, uint32_t slot) {
        g1_xyzz r;
        r.X = pt(lds, PX, slot); r.Y = pt(lds, PY, slot); r.ZZ = pt(lds, PZZ, slot); r.ZZZ = pt(lds, PZZZ, slot);
        return r;
    }
    TC_DEV static void point_set(uint8_t* lds, uint32_t slot, const g1_xyzz& p) {
        pt_set(lds, PX, slot, p.X); pt_set(lds, PY, slot, p.Y); pt_set(lds, PZZ, slot, p.ZZ); pt_set(lds, PZZZ, slot, p.ZZZ);
    }

    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t count = src.count(wg);
        if (ph == 0) {
            point_set(lds, lane, lane < count ? src.load(wg, lane) : xyzz_identity());
            return;
        }
        if (ph == PHASES - 1) {
            if (lane == 0) src.store(wg, point(lds, 0));
            return;
        }
        int q = ph - 1;
        int lv = q < 10 ? 0 : (q - 10) / 5 + 1, sub = q % 5;
        uint32_t stride = 1u << lv, npairs = (uint32_t)(NP / 2) >> lv;
        uint32_t wave = lane >> 6;
        uint32_t* flag_id = (uint32_t*)(lds + FLAG_BASE);      /* 0 regular, 1 keep a, 2 take b */
        uint32_t* flag_pz = flag_id + TP;                       /* same x */
        uint32_t* flag_rz = flag_pz + TP;                       /* same y */
        {
            uint32_t pr = (lane & 63u) + ((q >= 5 && q < 10) ? 64u : 0u);       /* the pair; its temporaries sit at lane & 63 */
            if (pr >= npairs) return;
            uint32_t a = pr * 2 * stride, b = a + stride;
            if (b >= count) return;                             /* nothing but identities from b on */
            pr &= 63u;
            if (sub == 0) {
                if (wave == 0) {
                    fp_t ZZa = pt(lds, PZZ, a), ZZb = pt(lds, PZZ, b);
                    flag_id[pr] = fe_is_zero(ZZb) ? 1u : fe_is_zero(ZZa) ? 2u : 0u;
                    tmp_set(lds, TU1, pr, fp_mul(pt(lds, PX, a), ZZb));
                } else if (wave == 1) {
                    tmp_set(lds, TU2, pr, fp_mul(pt(lds, PX, b), pt(lds, PZZ, a)));
                } else if (wave == 2) {
                    tmp_set(lds, TS1, pr, fp_mul(pt(lds, PY, a), pt(lds, PZZZ, b)));
                } else {
                    tmp_set(lds, TS2, pr, fp_mul(pt(lds, PY, b), pt(lds, PZZZ, a)));
                }
            } else if (sub == 1) {
                if (wave == 0) {
                    fp_t Pd = fp_sub(tmp(lds, TU2, pr), tmp(lds, TU1, pr));
                    flag_pz[pr] = fe_is_zero(Pd) ? 1u : 0u;
                    tmp_set(lds, TU2, pr, Pd);
                    tmp_set(lds, TPP, pr, fp_sqr(Pd));
                } else if (wave == 1) {
                    fp_t Rd = fp_sub(tmp(lds, TS2, pr), tmp(lds, TS1, pr));
                    flag_rz[pr] = fe_is_zero(Rd) ? 1u : 0u;
                    tmp_set(lds, TS2, pr, Rd);
                    tmp_set(lds, TRR, pr, fp_sqr(Rd));
                } else if (wave == 2) {
                    tmp_set(lds, TZA, pr, fp_mul(pt(lds, PZZ, a), pt(lds, PZZ, b)));
                } else {
                    tmp_set(lds, TZB, pr, fp_mul(pt(lds, PZZZ, a), pt(lds, PZZZ, b)));
                }
            } else {
                bool regular = flag_id[pr] == 0u && flag_pz[pr] == 0u;
                if (sub == 2) {
                    if (wave == 0) {
                        tmp_set(lds, TPPP, pr, fp_mul(tmp(lds, TU2, pr), tmp(lds, TPP, pr)));
                    } else if (wave == 1) {
                        tmp_set(lds, TQ, pr, fp_mul(tmp(lds, TU1, pr), tmp(lds, TPP, pr)));
                    } else if (wave == 2) {
                        fp_t ZZ3 = fp_mul(tmp(lds, TZA, pr), tmp(lds, TPP, pr));
                        if (regular) pt_set(lds, PZZ, a, ZZ3);
                    }
                } else if (sub == 3) {
                    if (wave == 0) {
                        fp_t Q = tmp(lds, TQ, pr);
                        fp_t X3 = fp_sub(fp_sub(fp_sub(tmp(lds, TRR, pr), tmp(lds, TPPP, pr)), Q), Q);
                        tmp_set(lds, TRR, pr, fp_mul(tmp(lds, TS2, pr), fp_sub(Q, X3)));
                        if (regular) pt_set(lds, PX, a, X3);
                    } else if (wave == 1) {
                        tmp_set(lds, TS1, pr, fp_mul(tmp(lds, TS1, pr), tmp(lds, TPPP, pr)));
                    } else if (wave == 2) {
                        fp_t ZZZ3 = fp_mul(tmp(lds, TZB, pr), tmp(lds, TPPP, pr));
                        if (regular) pt_set(lds, PZZZ, a, ZZZ3);
                    }
                } else if (wave == 0) {
                    if (regular) {
                        pt_set(lds, PY, a, fp_sub(tmp(lds, TRR, pr), tmp(lds, TS1, pr)));
                    } else if (flag_id[pr] == 2u) {
                        point_set(lds, a, point(lds, b));
                    } else if (flag_id[pr] == 0u) {             /* same x: the same point, or opposite ones */
                        point_set(lds, a, flag_rz[pr] ? xyzz_dbl32(point(lds, a)) : xyzz_identity());
                    }
                }
            }
        }
    }
};

/* ---- bucket reduction: sum_k k B_k --------------------------------------------------- */
/* Cooperative kernel (one workgroup = BLOCK consecutive entries of `in`), phases separated
 * by barriers.  For block g:  S_g = sum_j in[g BLOCK + j]  and
 * W_g = sum_j (j + 1) in[g BLOCK + j]  (suffix sums by doubling strides, then their sum). */
template <int BLOCK>
struct WeightedBlockSum {
    static constexpr int LOG = (BLOCK == 256) ? 8 : (BLOCK == 128) ? 7 : (BLOCK == 64) ? 6 : -1;
    static constexpr int PHASES = 1 + LOG + 1 + LOG + 1;
    static constexpr size_t LDS_BYTES = 2 * BLOCK * sizeof(g1_xyzz);
    const g1_xyzz* in;
    uint32_t n;                 /* entries of `in`; positions >= n count as the identity */
    g1_xyzz* out_w;             /* per block */
    g1_xyzz* out_s;             /* per block */
    const g1_xyzz* in2;         /* optional second array: blocks split .. read in2 from position 0 */
    uint32_t split;             /* first block that reads in2 (ignored when in2 is null) */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        g1_xyzz* buf0 = (g1_xyzz*)lds;
        g1_xyzz* buf1 = buf0 + BLOCK;
        if (ph == 0) {
            bool second = in2 && wg >= split;
            uint64_t i = (uint64_t)(second ? wg - split : wg) * BLOCK + lane;
            buf0[lane] = i < n ? (second ? in2[i] : in[i]) : xyzz_identity();
            return;
        }
        if (ph <= LOG) {                       /* suffix sums, ping-pong */
            int s = ph - 1;
            g1_xyzz* cur = (s & 1) ? buf1 : buf0;
            g1_xyzz* nxt = (s & 1) ? buf0 : buf1;
            uint32_t stride = 1u << s;
            g1_xyzz v = cur[lane];
            if (lane + stride < (uint32_t)BLOCK) v = xyzz_add(v, cur[lane + stride]);
            nxt[lane] = v;
            return;
        }
        g1_xyzz* cur = (LOG & 1) ? buf1 : buf0;     /* suffix sums live here now */
        if (ph == LOG + 1) {
            if (lane == 0) out_s[wg] = cur[0];
            return;
        }
        if (ph <= 2 * LOG + 1) {                     /* tree sum in place */
            int s = ph - (LOG + 2);
            uint32_t stride = 1u << s;
            if ((lane & (2 * stride - 1)) == 0) cur[lane] = xyzz_add(cur[lane], cur[lane + stride]);
            return;
        }
        if (lane == 0) out_w[wg] = cur[0];
    }
};

/* Bucket reduction of a window of 32768 buckets seen as a 128 x 256 matrix (bucket k = 256 h + l + 1).  With the
 * row sums R_h (the 256 buckets with that high part) and the column sums C_l (the 128 buckets with that low part),
 *     sum_k k B_k = 256 sum_h h R_h + sum_l (l + 1) C_l,
 * one plain addition per bucket and direction instead of a weighted scan over all of them. */
/* Launches with few windows (a lone commitment), where nothing but depth counts: every
 * sum is a cooperative sum whose additions are shared by the four waves of a workgroup (CoopReduce), and the
 * weights are taken bit by bit.  With R_h and C_l the row and column sums of the 128 x 256 bucket matrix,
 *     sum_k k B_k = sum_(j=0..8) 2^j X_j + 256 sum_(j=0..6) 2^j Y_j,
 *     X_j = sum of the C_l with bit j of l + 1 set,   Y_j = sum of the R_h with bit j of h set:
 * one launch for the 384 row and column sums, one for the 16 bit sums, 16 independent chains of at most 14
 * doublings, one sum of 16 points. */
struct RowColSrc {             /* workgroup (w, g): g < 128 row g, else column g - 128 */
    const g1_xyzz* bucket;     /* windows * 32768 */
    g1_xyzz* rows;             /* windows * 256 (128 used) */
    g1_xyzz* cols;             /* windows * 256 */
    TC_DEV uint32_t count(uint32_t wg) const { return wg % 384u < 128u ? 256u : 128u; }
    TC_DEV g1_xyzz load(uint32_t wg, uint32_t i) const {
        uint32_t w = wg / 384u, g = wg % 384u;
        const g1_xyzz* base = bucket + (uint64_t)w * 32768u;
        return g < 128u ? base[g * 256u + i] : base[i * 256u + (g - 128u)];
    }
    TC_DEV void store(uint32_t wg, const g1_xyzz& r) const {
        uint32_t w = wg / 384u, g = wg % 384u;
        if (g < 128u) rows[(uint64_t)w * 256u + g] = r; else cols[(uint64_t)w * 256u + (g - 128u)] = r;
    }
};
struct BitSumSrc {             /* workgroup (w, j): j < 9 the columns with bit j of l + 1, else the rows with bit j - 9 of h */
    const g1_xyzz* rows;
    const g1_xyzz* cols;
    g1_xyzz* out;              /* windows * 16 */
    TC_DEV uint32_t count(uint32_t wg) const { return wg % 16u < 9u ? 256u : 128u; }
    TC_DEV g1_xyzz load(uint32_t wg, uint32_t i) const {
        uint32_t w = wg / 16u, j = wg % 16u;
        if (j < 9u) return (((i + 1u) >> j) & 1u) ? cols[(uint64_t)w * 256u + i] : xyzz_identity();
        return ((i >> (j - 9u)) & 1u) ? rows[(uint64_t)w * 256u + i] : xyzz_identity();
    }
    TC_DEV void store(uint32_t wg, const g1_xyzz& r) const { out[wg] = r; }
};
/* lane (w, j): 2^j X_j for the columns, 2^(8 + j - 9) Y_(j-9) for the rows.  Up to 14 doublings in a row and only
 * 16 chains per window: the nine products of an XYZZ doubling are shared by the four waves of a workgroup in three
 * levels (V = (2Y)^2, A = X^2 | W = 2Y V, S = X V, (3A)^2, V ZZ | 3A (S - X3), W Y, W ZZZ), operands in LDS, a barrier
 * after every level and one more for the subtraction that ends the doubling; a chain that has done its own number
 * of doublings no longer takes the results.  ZZ = 0 (the identity) reproduces itself. */
struct BitSumScale {
    static constexpr int BLOCK = 256;
    static constexpr int MAX_DOUBLINGS = 14;
    enum { FX, FY, FZZ, FZZZ, FU, FV, FM, FW, FS, FMM, FT, FWY, FZZN, FZZZN, FX3, NFIELD };
    static constexpr size_t LDS_BYTES = (size_t)NFIELD * 3 * 64 * 16;
    static constexpr int PHASES = 1 + 4 * MAX_DOUBLINGS + 1;
    const g1_xyzz* in;
    uint32_t n;                /* chains: 16 per window */
    g1_xyzz* out;
    TC_DEV static uint32_t doublings(uint32_t t) {
        uint32_t j = t % 16u;
        return j < 9u ? j : j - 9u + 8u;
    }
    TC_DEV static fp_t ld(const uint8_t* lds, int f, uint32_t l) {
        const Quad16* q = (const Quad16*)lds;
        fp_t r;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            Quad16 t = q[(f * 3 + i) * 64 + l];
            r.l[4 * i] = t.v[0]; r.l[4 * i + 1] = t.v[1]; r.l[4 * i + 2] = t.v[2]; r.l[4 * i + 3] = t.v[3];
        }
        return r;
    }
    TC_DEV static void st(uint8_t* lds, int f, uint32_t l, const fp_t& x) {
        Quad16* q = (Quad16*)lds;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            Quad16 t;
            t.v[0] = x.l[4 * i]; t.v[1] = x.l[4 * i + 1]; t.v[2] = x.l[4 * i + 2]; t.v[3] = x.l[4 * i + 3];
            q[(f * 3 + i) * 64 + l] = t;
        }
    }
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t wave = lane >> 6, l = lane & 63u;
        uint32_t t = wg * 64u + l;
        bool live = t < n;
        if (ph == 0) {
            if (wave != 0) return;
            g1_xyzz p = live ? in[t] : xyzz_identity();
            st(lds, FX, l, p.X); st(lds, FY, l, p.Y); st(lds, FZZ, l, p.ZZ); st(lds, FZZZ, l, p.ZZZ);
            st(lds, FU, l, fp_dbl(p.Y));
            return;
        }
        if (ph == PHASES - 1) {
            if (wave != 0 || !live) return;
            g1_xyzz p;
            p.X = ld(lds, FX, l); p.Y = ld(lds, FY, l); p.ZZ = ld(lds, FZZ, l); p.ZZZ = ld(lds, FZZZ, l);
            out[t] = p;
            return;
        }
        uint32_t d = (uint32_t)(ph - 1) / 4u + 1u;          /* the d-th doubling is in the making */
        int level = (ph - 1) % 4;
        if (level == 0) {
            if (wave == 0) {
                st(lds, FV, l, fp_sqr_lat(ld(lds, FU, l)));
            } else if (wave == 1) {
                fp_t A = fp_sqr_lat(ld(lds, FX, l));
                st(lds, FM, l, fp_add(fp_dbl(A), A));
            }
        } else if (level == 1) {
            if (wave == 0) st(lds, FW, l, fp_mul_lat(ld(lds, FU, l), ld(lds, FV, l)));
            else if (wave == 1) st(lds, FS, l, fp_mul_lat(ld(lds, FX, l), ld(lds, FV, l)));
            else if (wave == 2) st(lds, FMM, l, fp_sqr_lat(ld(lds, FM, l)));
            else st(lds, FZZN, l, fp_mul_lat(ld(lds, FV, l), ld(lds, FZZ, l)));
        } else if (level == 2) {
            if (wave == 0) {
                fp_t S = ld(lds, FS, l);
                fp_t X3 = fp_sub(fp_sub(ld(lds, FMM, l), S), S);
                st(lds, FX3, l, X3);
                st(lds, FT, l, fp_mul_lat(ld(lds, FM, l), fp_sub(S, X3)));
            } else if (wave == 1) {
                st(lds, FWY, l, fp_mul_lat(ld(lds, FW, l), ld(lds, FY, l)));
            } else if (wave == 2) {
                st(lds, FZZZN, l, fp_mul_lat(ld(lds, FW, l), ld(lds, FZZZ, l)));
            }
        } else if (wave == 0 && live && d <= doublings(t)) {
            fp_t Y3 = fp_sub(ld(lds, FT, l), ld(lds, FWY, l));
            st(lds, FX, l, ld(lds, FX3, l));
            st(lds, FY, l, Y3);
            st(lds, FU, l, fp_dbl(Y3));
            st(lds, FZZ, l, ld(lds, FZZN, l));
            st(lds, FZZZ, l, ld(lds, FZZZN, l));
        }
    }
};
struct GroupSumSrc {           /* out[g] = sum of in[g * group .. (g + 1) * group), group <= 256 */
    const g1_xyzz* in;
    uint32_t group;
    g1_xyzz* out;
    TC_DEV uint32_t count(uint32_t) const { return group; }
    TC_DEV g1_xyzz load(uint32_t g, uint32_t i) const { return in[(uint64_t)g * group + i]; }
    TC_DEV void store(uint32_t g, const g1_xyzz& r) const { out[g] = r; }
};

/* one lane per window: 256 (W_R - S_R) + W_C */
struct RowColFinish {
    const g1_xyzz* w_rows;      /* sum_h (h + 1) R_h */
    const g1_xyzz* s_rows;      /* sum_h R_h */
    const g1_xyzz* w_cols;      /* sum_l (l + 1) C_l */
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t w) const {
        xyzz_acc t = acc_from(w_rows[w]);
        acc_add(t, acc_from(xyzz_neg(s_rows[w])));
        for (int i = 0; i < 8; ++i) acc_dbl(t);
        acc_add(t, acc_from(w_cols[w]));
        out[w] = acc_result(t);
    }
};

/* ---- many small windows: sum_k k B_k with one lane per row or column ---------------------------------------------
 * The row problems of a batch of openings end in tens of thousands of windows of 128 (or 256) buckets.  A window
 * is a 16 x 8 (16 x 16) matrix, k = cols h + l + 1:  sum_k k B_k = cols sum_h h R_h + sum_l (l + 1) C_l  over its row
 * sums R_h and column sums C_l.  StridedSums: one lane per row and one per column, all rows of all windows first and
 * the columns after them (the lanes of a wave then have equally many terms), the general addition expanded in place
 * as in AccXyzzFast, no LDS, nothing shared between lanes; a lane that meets equal or opposite sums enters itself in
 * a list that StridedRedo works off.  SmallWeighted: two lanes per window, the weighted sums by running sums
 * (run += X_i, total += run, from the far end); SmallFinish: one lane per window.
 * (Before: one wave per two windows summing through LDS with a call per product, at one wave per SIMD;
 * the 23 552 windows of the LLaMA2-7B-shaped openings 4.6 ms.) */
/* the sum of the terms that J.job hands lane t, to the slot it names: the loop of AccXyzzFast */
template <class Job>
TC_DEV void strided_sum_fast(const Job& J, uint32_t t) {
    uint64_t first, slot;
    uint32_t step, cnt;
    J.job(t, first, step, cnt, slot);
    g1_xyzz28 acc;
    bool have = false;
    for (uint32_t i = 0; i < cnt; ++i) {
        const g1_xyzz* at = J.in + (first + (uint64_t)i * step);
        /* four fifths of the 32768 buckets of a quantised activation are empty (its fp16 values are a coarse grid
         * away from zero): ZZ alone says so, a quarter of the point's bytes */
        if (fe_is_zero(at->ZZ)) continue;
        g1_xyzz p = *at;
        g1_xyzz28 q = xyzz28_from(p);
        if (!have) {
            acc = q;
            have = true;
            continue;
        }
        if (!acc_add_regular_expanded(acc, q)) {
            J.redo_list[atomic_add_u32(J.redo_count, 1u)] = t;
            return;
        }
    }
    g1_xyzz r;
    if (!have) {
        r = xyzz_identity();
    } else {
        r.X = fp28_to_fp_outlined(acc.X); r.Y = fp28_to_fp_outlined(acc.Y);
        r.ZZ = fp28_to_fp_outlined(acc.ZZ); r.ZZZ = fp28_to_fp_outlined(acc.ZZZ);
    }
    J.out[slot] = r;
}
/* the lanes that gave up, with the routine that settles every case */
template <class Job>
struct StridedRedo {
    Job J;
    uint32_t lanes;
    TC_DEV void operator()(uint32_t lane) const {
        for (uint32_t k = lane; k < *J.redo_count; k += lanes) {
            uint64_t first, slot;
            uint32_t step, cnt;
            J.job(J.redo_list[k], first, step, cnt, slot);
            xyzz_acc acc = acc_identity();
            for (uint32_t i = 0; i < cnt; ++i) acc_add(acc, acc_from(J.in[first + (uint64_t)i * step]));
            J.out[slot] = acc_result(acc);
        }
    }
};
struct StridedSums {
    const g1_xyzz* in;            /* n_windows * nb buckets */
    uint32_t nb;                  /* 128 or 256 */
    uint32_t n_windows;
    g1_xyzz* out;                 /* per window: 16 row sums, then nb / 16 column sums */
    uint32_t* redo_count;         /* zero before the launch */
    uint32_t* redo_list;          /* room for every lane */
    TC_HD uint32_t cols() const { return nb / 16u; }
    TC_HD uint64_t lanes() const { return (uint64_t)n_windows * (16u + cols()); }
    /* the terms of lane t: in[first + i * step], i < cnt, and where their sum goes */
    TC_HD void job(uint32_t t, uint64_t& first, uint32_t& step, uint32_t& cnt, uint64_t& slot) const {
        uint32_t c = cols(), n_rows = 16u * n_windows;
        if (t < n_rows) {
            uint32_t w = t / 16u, h = t % 16u;
            first = (uint64_t)w * nb + h * c; step = 1u; cnt = c;
            slot = (uint64_t)w * (16u + c) + h;
        } else {
            uint32_t u = t - n_rows, w = u / c, l = u % c;
            first = (uint64_t)w * nb + l; step = c; cnt = 16u;
            slot = (uint64_t)w * (16u + c) + 16u + l;
        }
    }
    TC_DEV void operator()(uint32_t t) const { strided_sum_fast(*this, t); }
};
/* The same for windows of 32768 buckets, a 128 x 256 matrix (k = 256 h + l + 1), in two levels so that the chip is
 * full and no lane has more than sixteen terms.  Level 1, per window: 2048 lanes for the sixteen pieces of each row,
 * 2048 for the eight pieces of each column (neighbouring lanes take neighbouring columns); level 2: 256 lanes for the
 * rows (the upper 128 have nothing to add and write the identity that WeightedBlockSum<256> expects there), 256 for
 * the columns.  (Before: four rows or columns per wave summed through LDS, a call per product: the 96 windows of the
 * LLaMA2-7B-shaped build 2.27 ms.) */
struct BigRowColSums {
    const g1_xyzz* in;            /* level 1: windows * 32768 buckets; level 2: windows * 4096 sums of level 1 */
    int level;
    uint32_t n_windows;
    g1_xyzz* out;                 /* level 1: windows * 4096; level 2: windows * 256 row sums, then windows * 256 column sums */
    uint32_t* redo_count;
    uint32_t* redo_list;
    TC_HD uint64_t lanes() const { return (uint64_t)n_windows * (level == 1 ? 4096u : 512u); }
    TC_HD void job(uint32_t t, uint64_t& first, uint32_t& step, uint32_t& cnt, uint64_t& slot) const {
        /* Lanes are numbered with the small magnitudes first, over all windows: the buckets of a quantised activation
         * are all full near zero and mostly empty further out (its fp16 values thin out), so a few lanes per window have
         * sixteen sums to add and most have none -- in window order those few chains started all through the launch,
         * one batch of resident waves after the other (1.2 ms); at its head they run side by side. */
        if (level == 1) {
            /* the rows 0 .. 15 of all windows, the columns' pieces over those rows, the other rows, the other pieces */
            const uint32_t r0 = 16u * 16u * n_windows, c0 = 256u * n_windows, r1 = 112u * 16u * n_windows;
            bool row = t < r0 || (t >= r0 + c0 && t < r0 + c0 + r1);
            if (row) {                            /* row h, piece sg: (h * windows + w) * 16 + sg within its class */
                uint32_t u = t < r0 ? t : t - r0 - c0, h0 = t < r0 ? 0u : 16u;
                uint32_t sg = u % 16u, hw = u / 16u, w = hw % n_windows, h = h0 + hw / n_windows;
                first = (uint64_t)w * 32768u + h * 256u + sg * 16u; step = 1u; cnt = 16u;
                slot = (uint64_t)w * 4096u + h * 16u + sg;
            } else {                              /* column l, piece sg: (sg * windows + w) * 256 + l within its class */
                uint32_t u = t < r0 + c0 ? t - r0 : t - r0 - c0 - r1, s0 = t < r0 + c0 ? 0u : 1u;
                uint32_t l = u % 256u, sw = u / 256u, w = sw % n_windows, sg = s0 + sw / n_windows;
                first = (uint64_t)w * 32768u + (uint64_t)sg * 16u * 256u + l; step = 256u; cnt = 16u;
                slot = (uint64_t)w * 4096u + 2048u + l * 8u + sg;
            }
        } else {
            uint32_t half = 256u * n_windows;
            if (t < half) {                       /* row h: t = h * windows + w */
                uint32_t w = t % n_windows, h = t / n_windows;
                first = (uint64_t)w * 4096u + h * 16u; step = 1u; cnt = h < 128u ? 16u : 0u;
                slot = (uint64_t)w * 256u + h;
            } else {
                uint32_t u = t - half, w = u / 256u, l = u % 256u;
                first = (uint64_t)w * 4096u + 2048u + l * 8u; step = 1u; cnt = 8u;
                slot = (uint64_t)half + u;
            }
        }
    }
    TC_DEV void operator()(uint32_t t) const { strided_sum_fast(*this, t); }
};
/* lane t < n_windows: sum_h h R_h of window t; lane n_windows + w: sum_l (l + 1) C_l of window w */
struct SmallWeighted {
    const g1_xyzz* sums;          /* per window: 16 row sums, then `cols` column sums */
    uint32_t cols, n_windows;
    g1_xyzz* out;                 /* [0, n_windows): the row part, [n_windows, 2 n_windows): the column part */
    TC_DEV void operator()(uint32_t t) const {
        bool rows = t < n_windows;
        uint32_t w = rows ? t : t - n_windows;
        const g1_xyzz* X = sums + (uint64_t)w * (16u + cols) + (rows ? 0u : 16u);
        uint32_t n = rows ? 16u : cols, last = rows ? 1u : 0u;      /* the row h = 0 has weight 0 */
        xyzz_acc run = acc_identity(), total = acc_identity();
        for (uint32_t i = n; i-- > last;) {
            acc_add(run, acc_from(X[i]));
            acc_add(total, run);
        }
        out[t] = acc_result(total);
    }
};
struct SmallFinish {             /* cols * (row part) + (column part) */
    const g1_xyzz* parts;
    uint32_t cols, n_windows;
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t w) const {
        xyzz_acc t = acc_from(parts[w]);
        for (uint32_t c = cols; c > 1u; c >>= 1) acc_dbl(t);
        acc_add(t, acc_from(parts[n_windows + w]));
        out[w] = acc_result(t);
    }
};

/* One lane per window: Wsum = sumW + BLOCK * (W2 - S2) where, over the G blocks of the window,
 * sumW = sum_g W_g, W2 = sum_g (g+1) S_g, S2 = sum_g S_g.  With G == 1: Wsum = W_0. */
struct WindowFinish {
    const g1_xyzz* w1;     /* W_g of stage 1, G per window (G == 1) or sum of them (stage 3 S) */
    const g1_xyzz* w2;     /* W of stage 2 per window */
    const g1_xyzz* s2;     /* S of stage 2 per window */
    int G, log_block;
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t w) const {
        if (G == 1) { out[w] = w1[w]; return; }
        xyzz_acc t = acc_from(w2[w]);
        acc_add(t, acc_from(xyzz_neg(s2[w])));
        for (int i = 0; i < log_block; ++i) acc_dbl(t);
        acc_add(t, acc_from(w1[w]));
        out[w] = acc_result(t);
    }
};
/* One lane per problem: Horner over its windows, result = sum_w 2^(c w) Wsum_w */
struct WindowCombine {
    const g1_xyzz* wsum;
    int W, c;
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t p) const {
        const g1_xyzz* ws = wsum + (uint64_t)p * W;
        if (W == 1) { out[p] = ws[0]; return; }
        xyzz_acc acc = acc_from(ws[W - 1]);
        for (int w = W - 2; w >= 0; --w) {
            for (int i = 0; i < c; ++i) acc_dbl(acc);
            acc_add(acc, acc_from(ws[w]));
        }
        out[p] = acc_result(acc);
    }
};

/* out[t] = 2^doublings * in[t]: the second half of a table whose high digits share the buckets of the low ones */
struct ShiftPoints {
    const g1_affine* in;
    int doublings;
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t t) const {
        xyzz_acc acc = acc_from(xyzz_from_affine(in[t]));
        for (int i = 0; i < doublings; ++i) acc_dbl(acc);
        out[t] = acc_result(acc);
    }
};

/* ---- normalisation: XYZZ -> affine (batched inversion) and canonical bytes ---------- */
/* Lane handles G consecutive points with one field inversion (Montgomery's trick).  The
 * running products are parked in out[i].x until the backward sweep overwrites them. */
struct BatchNormalize {
    const g1_xyzz* in;
    uint64_t n;
    uint32_t G;
    g1_affine* out;
    TC_DEV void operator()(uint32_t t) const {
        uint64_t lo = (uint64_t)t * G, hi = lo + G < n ? lo + G : n;
        if (lo >= hi) return;
        fp_t run = fe_one<FpParams>();
        for (uint64_t i = lo; i < hi; ++i) {
            out[i].x = run;                       /* product of z_lo .. z_{i-1} */
            if (!fe_is_zero(in[i].ZZ)) run = fp_mul(run, fp_mul(in[i].ZZ, in[i].ZZZ));
        }
        fp_t inv = fp_inv28(run);                    /* run != 0: product of non-zero values */
        for (uint64_t i = hi; i-- > lo;) {
            g1_xyzz p = in[i];
            if (fe_is_zero(p.ZZ)) {
                out[i] = affine_identity();
                continue;
            }
            fp_t zi = fp_mul(inv, out[i].x);       /* 1 / (ZZ_i ZZZ_i) */
            inv = fp_mul(inv, fp_mul(p.ZZ, p.ZZZ));
            out[i] = xyzz_to_affine_with_inv(p, zi);
        }
    }
};
struct ToCanonical {
    const g1_affine* in;
    uint32_t* out;          /* 24 words per point */
    TC_DEV void operator()(uint32_t t) const { affine_to_canonical(in[t], out + 24 * (uint64_t)t); }
};
struct ToCanonicalGather {   /* the same for points scattered over several arrays */
    const g1_affine* const* in;
    uint32_t* out;
    TC_DEV void operator()(uint32_t t) const { affine_to_canonical(*in[t], out + 24 * (uint64_t)t); }
};
struct PhiKernel {
    const g1_affine* in;
    fr_plain* out;
    TC_DEV void operator()(uint32_t t) const {
        fr_t v = phi_map(in[t]);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[t].l[i] = v.l[i];
    }
};

/* ---- fixed-base window tables -------------------------------------------------------- */
/* Table layout: entry ((k * FB_W + w) * FB_NB + j - 1) = j * 2^(c w) * B_k, affine, j = 1..2^(c-1),
 * c = FB_C (16: 16 windows of 32768 entries, 50 MB per base). */
#ifndef TC_FB_C
#define TC_FB_C 16             /* window width; the host-emulation build of the tests uses 8 */
#endif
constexpr int FB_C = TC_FB_C;
constexpr int FB_W = 256 / FB_C;
constexpr uint32_t FB_NB = 1u << (FB_C - 1);
constexpr uint32_t FB_CHUNK = 64;

struct FbWindowBases {         /* lane k: 2^(c w) B_k for every window w */
    const g1_affine* bases;
    g1_xyzz* out;              /* nbases * FB_W */
    TC_DEV void operator()(uint32_t k) const {
        g1_xyzz p = xyzz_from_affine(bases[k]);
        for (int w = 0; w < FB_W; ++w) {
            out[(uint64_t)k * FB_W + w] = p;
            if (w + 1 < FB_W)
                for (int i = 0; i < FB_C; ++i) p = xyzz_dbl(p);
        }
    }
};
struct FbChunkFill {           /* lane (bw, chunk): multiples j0 .. j0 + 63 of window base bw */
    const g1_affine* wbase;    /* affine window bases, `count` of them starting at bw0 */
    uint32_t bw0;
    g1_xyzz* out;              /* count * FB_NB */
    TC_DEV void operator()(uint32_t t) const {
        uint32_t chunks = FB_NB / FB_CHUNK;
        uint32_t bw = t / chunks, ch = t % chunks;
        g1_affine b = wbase[bw0 + bw];
        uint32_t j0 = ch * FB_CHUNK + 1;
        g1_xyzz acc = xyzz_mul_affine(&j0, 17, b);
        uint64_t base = (uint64_t)bw * FB_NB + (j0 - 1);
        for (uint32_t i = 0; i < FB_CHUNK; ++i) {
            out[base + i] = acc;
            acc = xyzz_madd(acc, b);
        }
    }
};

/* acc += sum_w digit_w(v) * table[(k, w)] for a canonical Fr value v */
TC_HD void fb_mul_accumulate(xyzz_acc& acc, const g1_affine* table, uint32_t k, const uint32_t* v) {
    uint32_t carry = 0;
    for (int w = 0; w < FB_W; ++w) {
        int32_t d = fr_window_digit(v, w, FB_C, carry);
        if (d) acc_madd(acc, table[((uint64_t)k * FB_W + w) * FB_NB + (uint32_t)(d < 0 ? -d : d) - 1u], d < 0);
    }
}
/* windows 2h and 2h + 1 only: digit_{2h}(v) table[(k, 2h)] + digit_{2h+1}(v) table[(k, 2h + 1)].  The digits are
 * found first (their carries come from the windows below), so that the two additions sit outside any loop
 * whose length differs between the lanes of a wave. */
TC_HD g1_xyzz fb_window_pair(const g1_affine* table, uint32_t k, const uint32_t* v, uint32_t h) {
    uint32_t carry = 0;
    int32_t d0 = 0, d1 = 0;
    for (int w = 0; w <= (int)(2 * h + 1); ++w) {
        int32_t d = fr_window_digit(v, w, FB_C, carry);
        if (w == (int)(2 * h)) d0 = d;
        if (w == (int)(2 * h + 1)) d1 = d;
    }
    xyzz_acc acc = acc_identity();
    for (int j = 0; j < 2; ++j) {
        int32_t d = j ? d1 : d0;
        g1_affine p = affine_identity();
        if (d) p = table[((uint64_t)k * FB_W + 2 * h + j) * FB_NB + (uint32_t)(d < 0 ? -d : d) - 1u];
        acc_madd(acc, p, d < 0);
    }
    return acc_result(acc);
}
/* same for a small signed integer |d| <= 2^15 (one lookup when the window is 16 bits wide) */
TC_HD void fb_small_accumulate(xyzz_acc& acc, const g1_affine* table, uint32_t k, int32_t d) {
    if (!d) return;
    uint32_t mag = (uint32_t)(d < 0 ? -d : d);
    if (FB_C == 16) {
        acc_madd(acc, table[((uint64_t)k * FB_W) * FB_NB + mag - 1u], d < 0);
        return;
    }
    uint32_t v[8] = {mag, 0, 0, 0, 0, 0, 0, 0};
    uint32_t carry = 0;
    for (int w = 0; w * FB_C < 24; ++w) {
        int32_t dw = fr_window_digit(v, w, FB_C, carry);
        if (dw) {
            bool negative = (dw < 0) != (d < 0);
            acc_madd(acc, table[((uint64_t)k * FB_W + w) * FB_NB + (uint32_t)(dw < 0 ? -dw : dw) - 1u], negative);
        }
    }
}

/* ---- SRS generation (Def. 4.1 Setup, Lagrange image) ---------------------------------- */
struct ShapeInfo {
    int m;
    uint32_t d[4];
};
TC_HD void unflatten(uint64_t f, const ShapeInfo& s, int first_axis, uint32_t* idx) {
    for (int j = s.m - 1; j >= first_axis; --j) {
        idx[j] = (uint32_t)(f % s.d[j]);
        f /= s.d[j];
    }
}
struct SrsGen {                /* lane i: S^(a)[i] = [prod_{j>=a} l_j[i_j]] G */
    ShapeInfo shape;
    int first_axis;
    const fr_t* ell;           /* Montgomery Lagrange values, axes concatenated */
    uint32_t ell_off[4];
    const g1_affine* gtable;   /* fixed-base table of G (one base) */
    uint64_t i0;               /* first point of this launch */
    g1_xyzz* out;              /* indexed from 0 for point i0 */
    TC_DEV void operator()(uint32_t t) const {
        uint64_t i = i0 + t;
        uint32_t idx[4];
        unflatten(i, shape, first_axis, idx);
        fr_t s = ell[ell_off[first_axis] + idx[first_axis]];
        for (int j = first_axis + 1; j < shape.m; ++j) s = fr_mul(s, ell[ell_off[j] + idx[j]]);
        fr_t plain = fe_to_plain(s);
        xyzz_acc acc = acc_identity();
        fb_mul_accumulate(acc, gtable, 0, plain.l);
        out[t] = acc_result(acc);
    }
};

/* Factors of the opening table of the leading axis: lane kappa computes
 *     g(kappa) = sum_(k != kappa) l_k(tau) / (zeta_k - zeta_kappa),     zeta_k - zeta_kappa = k - kappa,
 * so that U[kappa, t] = sum_(k != kappa) S[k, t] / (zeta_k - zeta_kappa) = [g(kappa) prod_(j > 0) l_j[t_j]] G comes out of
 * the SRS generator with g in the place of the leading axis' Lagrange values. */
struct OpenTableFactors {
    const fr_t* ell;           /* l_k(tau) of the leading axis, Montgomery */
    const fr_t* inv_int;       /* 1 / j, j = 1 .. d-1 */
    uint32_t d;
    fr_t* out;
    TC_DEV void operator()(uint32_t kappa) const {
        fr_t pos = fe_zero<FrParams>(), neg = fe_zero<FrParams>();
        for (uint32_t k = 0; k < d; ++k) {
            if (k == kappa) continue;
            fr_t t = fr_mul(ell[k], inv_int[k > kappa ? k - kappa : kappa - k]);
            if (k > kappa) pos = fr_add(pos, t); else neg = fr_add(neg, t);
        }
        out[kappa] = fr_sub(pos, neg);
    }
};

/* ---- Terkle node commitments ----------------------------------------------------------- */
struct TreeGeom {
    int m;
    uint32_t node[4];          /* node shape */
    uint32_t below[4];         /* grid of the level below (payload grid for level 0) */
    uint32_t grid[4];          /* grid of this level */
    uint32_t B;                /* arity */
};
/* flat index in the level below of child k (flat in node shape) of node a (flat in grid); -1 if outside */
TC_HD int64_t child_index(const TreeGeom& g, uint64_t a, uint32_t k) {
    uint32_t ai[4], ki[4];
    for (int j = g.m - 1; j >= 0; --j) {
        ai[j] = (uint32_t)(a % g.grid[j]);
        a /= g.grid[j];
        ki[j] = k % g.node[j];
        k /= g.node[j];
    }
    uint64_t f = 0;
    for (int j = 0; j < g.m; ++j) {
        uint64_t p = (uint64_t)ai[j] * g.node[j] + ki[j];
        if (p >= g.below[j]) return -1;
        f = f * g.below[j] + p;
    }
    return (int64_t)f;
}
/* bottom level of an entries tree: lane = node, children are small integers */
struct NodeCommitSmall {
    TreeGeom g;
    const void* payload;
    int dtype;
    const g1_affine* table;
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t a) const {
        xyzz_acc acc = acc_identity();
        for (uint32_t k = 0; k < g.B; ++k) {
            int64_t f = child_index(g, a, k);
            if (f < 0) continue;
            fb_small_accumulate(acc, table, k, small_scalar(payload, dtype, (uint64_t)f));
        }
        out[a] = acc_result(acc);
    }
};
/* the same for a bottom level of very few nodes: every child its own slot of a cooperative sum */
struct NodeSmallSrc {
    TreeGeom g;
    const void* payload;
    int dtype;
    const g1_affine* table;
    g1_xyzz* out;
    TC_DEV uint32_t count(uint32_t) const { return g.B < 256u ? g.B : 256u; }
    TC_DEV g1_xyzz load(uint32_t node, uint32_t i) const {
        xyzz_acc acc = acc_identity();
        for (uint32_t k = i; k < g.B; k += 256) {
            int64_t f = child_index(g, node, k);
            if (f >= 0) fb_small_accumulate(acc, table, k, small_scalar(payload, dtype, (uint64_t)f));
        }
        return acc_result(acc);
    }
    TC_DEV void store(uint32_t node, const g1_xyzz& r) const { out[node] = r; }
};
/* upper levels: lane = (node, child); the child's value is phi of the commitment below */
struct NodeCommitFr {
    TreeGeom g;
    const fr_plain* below;
    const g1_affine* table;
    g1_xyzz* out;               /* n_nodes * B partial sums */
    TC_DEV void operator()(uint32_t t) const {
        uint32_t a = t / g.B, k = t % g.B;
        int64_t f = child_index(g, a, k);
        xyzz_acc acc = acc_identity();
        if (f >= 0) fb_mul_accumulate(acc, table, k, below[f].l);
        out[t] = acc_result(acc);
    }
};
/* upper levels, arity a power of two <= 64: a lane commits FB_W >> logH consecutive windows of one child
 * (B << logH <= 64 lanes per node, BLOCK / (B << logH) nodes per workgroup), then the partial sums of a node are
 * added pairwise through LDS.  Large levels take four waves per workgroup, so that most waves skip the later
 * halving steps; small ones a single wave.  logH = 0 (one lane per child) does the least work in
 * total; a level of few nodes is bound by the depth of one lane's work instead and takes logH > 0. */
template <int BLOCK>
struct NodeCommitFrCoop {
    static constexpr size_t LDS_BYTES = BLOCK * sizeof(g1_xyzz);
    static constexpr int PHASES = 8;         /* 1 + log2(64) + 1 */
    TreeGeom g;
    const fr_plain* below;
    const g1_affine* table;
    uint64_t n_nodes;
    int logB, logH;
    g1_xyzz* out;               /* n_nodes */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        g1_xyzz* buf = (g1_xyzz*)lds;
        int logL = logB + logH;
        uint64_t t = (uint64_t)wg * BLOCK + lane;
        uint64_t a = t >> logL;
        uint32_t r = (uint32_t)(t & ((1u << logL) - 1u));
        if (ph == 0) {
            uint32_t k = r >> logH, h = r & ((1u << logH) - 1u);
            xyzz_acc acc = acc_identity();
            if (a < n_nodes) {
                int64_t f = child_index(g, a, k);
                if (f >= 0) {
                    const uint32_t* v = below[f].l;
                    int per = FB_W >> logH, w0 = (int)h * per;
                    uint32_t carry = 0;
                    for (int w = 0; w < w0; ++w) (void)fr_window_digit(v, w, FB_C, carry);     /* carry into the first window */
                    for (int j = 0; j < per; ++j) {            /* the same trip count in every lane */
                        int32_t d = fr_window_digit(v, w0 + j, FB_C, carry);
                        if (d) acc_madd(acc, table[((uint64_t)k * FB_W + w0 + j) * FB_NB + (uint32_t)(d < 0 ? -d : d) - 1u], d < 0);
                    }
                }
            }
            buf[lane] = acc_result(acc);
            return;
        }
        /* pairwise sums, the active lanes packed to the front of the workgroup: whole waves drop out as the
         * number of additions halves */
        uint32_t per_node = 1u << logL;
        if (ph <= logL) {
            uint32_t half = per_node >> ph;
            if (lane < ((uint32_t)BLOCK >> ph)) {
                uint32_t at = (lane / half) * per_node + lane % half;
                buf[at] = xyzz_add(buf[at], buf[at + half]);
            }
            return;
        }
        if (ph == logL + 1 && lane < (uint32_t)BLOCK / per_node) {
            uint64_t node = (uint64_t)wg * (BLOCK / per_node) + lane;
            if (node < n_nodes) out[node] = buf[lane * per_node];
        }
    }
};
/* levels of very few nodes: a node is the sum of its B * FB_W (child, window) table points */
struct NodeWindowSrc {
    TreeGeom g;
    const fr_plain* below;
    const g1_affine* table;
    g1_xyzz* out;               /* n_nodes */
    TC_DEV uint32_t count(uint32_t) const { return g.B * (uint32_t)FB_W < 256u ? g.B * (uint32_t)FB_W : 256u; }
    TC_DEV g1_xyzz load(uint32_t node, uint32_t i) const {
        g1_xyzz acc = xyzz_identity();
        for (uint32_t idx = i; idx < g.B * (uint32_t)FB_W; idx += 256) {
            uint32_t k = idx / (uint32_t)FB_W, w = idx % (uint32_t)FB_W;
            int64_t f = child_index(g, node, k);
            if (f < 0) continue;
            const uint32_t* v = below[f].l;
            uint32_t carry = 0;
            int32_t d = 0;
            for (uint32_t x = 0; x <= w; ++x) d = fr_window_digit(v, (int)x, FB_C, carry);
            if (!d) continue;
            g1_affine p = table[((uint64_t)k * FB_W + w) * FB_NB + (uint32_t)(d < 0 ? -d : d) - 1u];
            if (d < 0) p.y = fp_neg(p.y);
            acc = xyzz_madd32(acc, p);
        }
        return acc;
    }
    TC_DEV void store(uint32_t node, const g1_xyzz& r) const { out[node] = r; }
};
/* out[i] = sum of in[i * group .. (i + 1) * group) */
struct SumGroups {
    const g1_xyzz* in;
    uint32_t group;
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t t) const {
        const g1_xyzz* p = in + (uint64_t)t * group;
        xyzz_acc acc = acc_from(p[0]);
        for (uint32_t i = 1; i < group; ++i) acc_add(acc, acc_from(p[i]));
        out[t] = acc_result(acc);
    }
};
/* out[t] = sum of segment t of `in`: the elements in[off[t] * scale .. off[t + 1] * scale) */
struct SegmentSrc {
    const g1_xyzz* in;
    const uint32_t* off;
    uint32_t scale;
    g1_xyzz* out;
    TC_DEV uint32_t count(uint32_t t) const {
        uint64_t len = (uint64_t)(off[t + 1] - off[t]) * scale;
        return len < 256 ? (uint32_t)len : 256u;
    }
    TC_DEV g1_xyzz load(uint32_t t, uint32_t i) const {
        uint64_t lo = (uint64_t)off[t] * scale, hi = (uint64_t)off[t + 1] * scale;
        g1_xyzz acc = in[lo + i];
        for (uint64_t x = lo + i + 256; x < hi; x += 256) acc = xyzz_add32(acc, in[x]);
        return acc;
    }
    TC_DEV void store(uint32_t t, const g1_xyzz& r) const { out[t] = r; }
};

/* ---- Open: quotient values on the grid (Algorithm 1 in evaluation form) ----------------- */
/* Along one axis of length d with the opening at position kap, for every line t of the slice:
 *   q[k] = (g[k] - g[kap]) / (zeta_k - zeta_kap)            k != kap
 *   q[kap] = - sum_{k != kap} (beta_k / beta_kap) q[k]       (value of the same polynomial at zeta_kap)
 * with zeta_k = k + 1 and beta the barycentric weights of App. C. */
struct AxisTables {
    const fr_t* inv_int;     /* inv_int[j] = 1 / j (Montgomery), j = 1..d-1; entry 0 unused */
    const fr_t* beta;        /* beta_k (Montgomery) */
    const fr_t* beta_inv;    /* 1 / beta_k */
};
TC_HD fr_t scalar_as_fr(const void* s, int dtype, uint64_t i) {
    if (dtype == DT_FR) return fe_from_limbs<FrParams>(((const fr_plain*)s)[i].l);
    return fe_from_i32<FrParams>(small_scalar(s, dtype, i));
}
struct QuotientRows {        /* lane (k, t), k != kap */
    const void* scalars;
    int dtype;
    uint64_t offset;         /* start of the slice */
    uint32_t d, kap;
    uint64_t inner;
    AxisTables ax;
    fr_plain* q;             /* d * inner */
    TC_DEV void operator()(uint32_t lane) const {
        uint32_t k = (uint32_t)(lane / inner);
        uint64_t t = lane % inner;
        if (k == kap) return;
        fr_t num = fr_sub(scalar_as_fr(scalars, dtype, offset + (uint64_t)k * inner + t),
                          scalar_as_fr(scalars, dtype, offset + (uint64_t)kap * inner + t));
        uint32_t dist = k > kap ? k - kap : kap - k;
        fr_t v = fr_mul(num, ax.inv_int[dist]);
        if (k < kap) v = fr_neg(v);
        fr_t plain = fe_to_plain(v);
#pragma unroll
        for (int i = 0; i < 8; ++i) q[(uint64_t)k * inner + t].l[i] = plain.l[i];
    }
};
/* q[kap, t] = -(1/beta_kap) sum_{k != kap} beta_k q[k, t], in two steps so that a single line (inner = 1)
 * of thousands of entries is not one serial chain: lane (chunk, t) sums a chunk of k's, then lane t
 * adds the chunk sums. */
struct QuotientKappaPartial {
    uint32_t d, kap, chunks;
    uint64_t inner;
    AxisTables ax;
    const fr_plain* q;
    fr_t* partial;             /* chunks * inner, Montgomery */
    TC_DEV void operator()(uint32_t lane) const {
        uint32_t ch = (uint32_t)(lane / inner);
        uint64_t t = lane % inner;
        uint32_t per = (d + chunks - 1) / chunks;
        uint32_t k0 = ch * per, k1 = k0 + per < d ? k0 + per : d;
        fr_t acc = fe_zero<FrParams>();
        for (uint32_t k = k0; k < k1; ++k) {
            if (k == kap) continue;
            fr_t qv = fe_from_limbs<FrParams>(q[(uint64_t)k * inner + t].l);
            acc = fr_add(acc, fr_mul(ax.beta[k], qv));
        }
        partial[(uint64_t)ch * inner + t] = acc;
    }
};
struct QuotientKappaRow {    /* lane t */
    uint32_t kap, chunks;
    uint64_t inner;
    AxisTables ax;
    const fr_t* partial;
    fr_plain* q;
    TC_DEV void operator()(uint32_t t) const {
        fr_t acc = partial[t];
        for (uint32_t ch = 1; ch < chunks; ++ch) acc = fr_add(acc, partial[(uint64_t)ch * inner + t]);
        acc = fr_neg(fr_mul(acc, ax.beta_inv[kap]));
        fr_t plain = fe_to_plain(acc);
#pragma unroll
        for (int i = 0; i < 8; ++i) q[(uint64_t)kap * inner + t].l[i] = plain.l[i];
    }
};
/* Open along an axis with many lines per row (a leading axis of a large tensor), small-integer data:
 *   pi = sum_{k != kap} c_k R_k + sum_t q[kap, t] S[kap, t],   c_k = 1 / (zeta_k - zeta_kap),
 *   R_k = sum_t (T[k, t] - T[kap, t]) S[k, t]   (one small-scalar problem per row, 17-bit numerators),
 * so the bulk of the work is two 9-bit digits per entry instead of sixteen 16-bit windows. */
struct RowWeights {            /* plain c_k: lane j for the j-th row other than kap, or (all_rows) lane k for row k, 0 at kap */
    AxisTables ax;
    uint32_t kap;
    int all_rows;
    fr_plain* out;
    TC_DEV void operator()(uint32_t j) const {
        uint32_t k = all_rows ? j : (j < kap ? j : j + 1);
        fr_t plain = fe_zero<FrParams>();
        if (k != kap) {
            uint32_t dist = k > kap ? k - kap : kap - k;
            fr_t c = ax.inv_int[dist];
            if (k < kap) c = fr_neg(c);
            plain = fe_to_plain(c);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) out[j].l[i] = plain.l[i];
    }
};
struct KappaWeights {          /* lane k: beta_k c_k in Montgomery form (0 for k = kap) */
    AxisTables ax;
    uint32_t kap;
    fr_t* out;
    TC_DEV void operator()(uint32_t k) const {
        if (k == kap) { out[k] = fe_zero<FrParams>(); return; }
        uint32_t dist = k > kap ? k - kap : kap - k;
        fr_t w = fr_mul(ax.beta[k], ax.inv_int[dist]);
        out[k] = k < kap ? fr_neg(w) : w;
    }
};
/* 320-bit accumulator for sums of (small integer) x (Montgomery-form Fr value): no reduction per term */
struct Wide320 {
    uint32_t l[10];
};
/* value mod r, keeping the Montgomery factor of the summands: lo R / R + hi R^2 / R = lo + hi 2^256 */
TC_HD fr_t wide_reduce(const Wide320& a) {
    fr_t lo, hi, one, r2;
#pragma unroll
    for (int i = 0; i < 8; ++i) { lo.l[i] = a.l[i]; hi.l[i] = i < 2 ? a.l[8 + i] : 0u; one.l[i] = FrParams::ONE[i]; r2.l[i] = FrParams::R2[i]; }
    return fr_add(fr_mul(lo, one), fr_mul(hi, r2));
}
struct KappaRowDirect {        /* lane t: q[kap, t] = -(1/beta_kap) sum_{k != kap} beta_k c_k (T[k,t] - T[kap,t]) */
    const void* scalars;
    int dtype;
    uint64_t offset;
    uint32_t d, kap;
    uint64_t inner;
    AxisTables ax;
    const fr_t* wk;            /* KappaWeights */
    fr_plain* q;               /* inner values */
    TC_DEV void operator()(uint32_t t) const {
        int32_t gk = small_scalar(scalars, dtype, offset + (uint64_t)kap * inner + t);
        /* limb by limb, without carries between the terms: a term adds less than 2^49 to a limb's sum (a 32-bit limb
         * of the weight times a numerator of at most 17 bits), so 2^14 terms fit 64 bits; positive and negative
         * numerators apart, every multiply-add independent of the others and no branch in the loop */
        uint64_t sp[8], sn[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { sp[i] = 0; sn[i] = 0; }
        Wide320 pos, neg;
#pragma unroll
        for (int i = 0; i < 10; ++i) { pos.l[i] = 0; neg.l[i] = 0; }
        for (uint32_t k0 = 0; k0 < d; k0 += 8192u) {              /* sums are folded in before they could overflow */
            uint32_t k1 = k0 + 8192u < d ? k0 + 8192u : d;
#pragma unroll 4
            for (uint32_t k = k0; k < k1; ++k) {
                int32_t num = small_scalar(scalars, dtype, offset + (uint64_t)k * inner + t) - gk;
                if (k == kap) num = 0;
                uint32_t up = num > 0 ? (uint32_t)num : 0u, dn = num < 0 ? (uint32_t)(-num) : 0u;
                const fr_t w = wk[k];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    sp[i] += (uint64_t)w.l[i] * up;
                    sn[i] += (uint64_t)w.l[i] * dn;
                }
            }
            uint64_t cp = 0, cn = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                cp += (sp[i] & 0xFFFFFFFFull) + pos.l[i];
                cn += (sn[i] & 0xFFFFFFFFull) + neg.l[i];
                pos.l[i] = (uint32_t)cp;
                neg.l[i] = (uint32_t)cn;
                cp = (cp >> 32) + (sp[i] >> 32);
                cn = (cn >> 32) + (sn[i] >> 32);
                sp[i] = 0;
                sn[i] = 0;
            }
            cp += pos.l[8];
            cn += neg.l[8];
            pos.l[8] = (uint32_t)cp;
            neg.l[8] = (uint32_t)cn;
            pos.l[9] += (uint32_t)(cp >> 32);
            neg.l[9] += (uint32_t)(cn >> 32);
        }
        fr_t acc = fr_sub(wide_reduce(pos), wide_reduce(neg));
        acc = fr_neg(fr_mul(acc, ax.beta_inv[kap]));
        fr_t plain = fe_to_plain(acc);
#pragma unroll
        for (int i = 0; i < 8; ++i) q[t].l[i] = plain.l[i];
    }
};
/* ---- halving the scalars of a short full-width problem with the curve endomorphism -------------------------------
 * (x, y) -> (beta x, y) multiplies a point of the group by lambda, a root of X^2 + X + 1 mod r of 128 bits.  With
 * k = k1 + k2 lambda, 0 <= k1 < lambda and k2 < 2^128 (k < r < lambda^2 + lambda + 1), the term [k] P becomes
 * [k1] P + [k2] (beta x, y): twice the terms, half the windows, and -- what it is done for -- half the chain of
 * doublings that combines the windows of a problem, which two waves walk alone at the end of a batch of openings. */
TC_HD void glv_split128(const uint32_t k[8], uint32_t k1[4], uint32_t k2[4]) {
    const uint64_t lam_lo = (uint64_t)GLV_LAMBDA[0] | ((uint64_t)GLV_LAMBDA[1] << 32);
    const uint64_t lam_hi = (uint64_t)GLV_LAMBDA[2] | ((uint64_t)GLV_LAMBDA[3] << 32);
    /* the upper half of k is below 2^127 <= lambda (k < r < 2^255): the long division starts with it as the remainder */
    uint64_t r_lo = (uint64_t)k[4] | ((uint64_t)k[5] << 32), r_hi = (uint64_t)k[6] | ((uint64_t)k[7] << 32), q_lo = 0, q_hi = 0;
    for (int i = 127; i >= 0; --i) {
        bool top = (r_hi >> 63) != 0;
        r_hi = (r_hi << 1) | (r_lo >> 63);
        r_lo = (r_lo << 1) | (uint64_t)((k[i >> 5] >> (i & 31)) & 1u);
        if (top || r_hi > lam_hi || (r_hi == lam_hi && r_lo >= lam_lo)) {
            uint64_t borrow = r_lo < lam_lo ? 1u : 0u;      /* with `top` set the value is 2^128 + r, still >= lambda */
            r_lo -= lam_lo;
            r_hi -= lam_hi + borrow;
            if (i < 64) q_lo |= 1ull << i;
            else q_hi |= 1ull << (i - 64);
        }
    }
    k1[0] = (uint32_t)r_lo; k1[1] = (uint32_t)(r_lo >> 32); k1[2] = (uint32_t)r_hi; k1[3] = (uint32_t)(r_hi >> 32);
    k2[0] = (uint32_t)q_lo; k2[1] = (uint32_t)(q_lo >> 32); k2[2] = (uint32_t)q_hi; k2[3] = (uint32_t)(q_hi >> 32);
}
struct GlvExpand {           /* lane t: term t of the problem -> terms t and n + t of the expanded one */
    const g1_affine* pts;
    const fr_plain* k;
    uint64_t n;
    g1_affine* pts2;         /* 2 n points */
    fr_plain* k2;            /* 2 n scalars below 2^128 */
    TC_DEV void operator()(uint32_t t) const {
        g1_affine p = pts[t];
        pts2[t] = p;
        if (!affine_is_identity(p)) {
            fp_t beta;
#pragma unroll
            for (int i = 0; i < 12; ++i) beta.l[i] = GLV_BETA[i];
            p.x = fp_mul(p.x, beta);
        }
        pts2[n + t] = p;
        fr_plain lo, hi;
        glv_split128(k[t].l, lo.l, hi.l);
#pragma unroll
        for (int i = 4; i < 8; ++i) { lo.l[i] = 0; hi.l[i] = 0; }
        k2[t] = lo;
        k2[n + t] = hi;
    }
};
/* Many small jobs of one kind in one launch: job j owns the lanes first[j] .. first[j + 1] and runs its own
 * functor on them (the openings of a batch each have their own axes, positions and buffers). */
template <class F>
struct JobList {
    const F* jobs;
    const uint64_t* first;     /* njobs + 1 */
    uint32_t njobs;
    TC_DEV void operator()(uint32_t lane) const {
        uint32_t lo = 0, hi = njobs;
        while (hi - lo > 1) {
            uint32_t mid = (lo + hi) / 2;
            if (first[mid] <= lane) lo = mid;
            else hi = mid;
        }
        jobs[lo]((uint32_t)(lane - first[lo]));
    }
};
struct FillIdentity {
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t t) const { out[t] = xyzz_identity(); }
};
/* out = res[a] (+ res[b] when b >= 0) (- sub[c] when c >= 0): where the proof elements of a batch of openings end up */
struct CollectResult {
    const g1_xyzz* res;
    int32_t a, b;
    const g1_xyzz* sub;
    int32_t c;
    g1_xyzz* out;
    TC_DEV void operator()(uint32_t) const {
        g1_xyzz r = b >= 0 ? xyzz_add(res[a], res[b]) : res[a];
        if (c >= 0) r = xyzz_add(r, xyzz_neg(sub[c]));
        *out = r;
    }
};

/* y = e(T[f]) as canonical bytes */
struct FetchScalar {
    const void* scalars;
    int dtype;
    uint64_t f;
    fr_plain* out;
    TC_DEV void operator()(uint32_t) const {
        fr_t plain = fe_to_plain(scalar_as_fr(scalars, dtype, f));
#pragma unroll
        for (int i = 0; i < 8; ++i) out[0].l[i] = plain.l[i];
    }
};

/* ---- Terkle openings of node tensors (small shapes, fixed-base tables) ------------------- */
struct NodeOpenJob {           /* one (path, level) */
    uint64_t node;             /* flat node index in the level grid */
    uint32_t kappa[4];         /* child multi-index */
    int level;                 /* 0 = bottom (children are payload entries) */
    uint32_t term0;            /* first output slot of this job */
};
struct LevelView {             /* what a node's children are */
    TreeGeom g;
    const void* payload;       /* level 0 of an entries tree */
    int dtype;
    const fr_plain* below;     /* upper levels: phi values of the level below */
};
constexpr int MAX_LEVELS = 16;
struct NodeOpenTerms {         /* lane (job, axis, term, window pair): two windows of one quotient value times its suffix-SRS point */
    const NodeOpenJob* jobs;
    LevelView lv[MAX_LEVELS];
    ShapeInfo node;            /* node shape */
    uint32_t terms_per_job;    /* sum_a prod_{j>=a} d_j */
    uint32_t axis_first[5];    /* first term of axis a within a job */
    AxisTables ax[4];
    const g1_affine* table[4]; /* fixed-base tables of S^(a) */
    int logH;                  /* log2(FB_W / 2) window pairs per term */
    g1_xyzz* out;              /* jobs * terms_per_job << logH */
    fr_plain* y_out;           /* per job: the opened value */

    TC_DEV fr_t child_value(const LevelView& v, uint64_t a, const uint32_t* k) const {
        uint32_t kf = 0;
        for (int j = 0; j < node.m; ++j) kf = kf * node.d[j] + k[j];
        int64_t f = child_index(v.g, a, kf);
        if (f < 0) return fe_zero<FrParams>();
        if (v.payload) return fe_from_i32<FrParams>(small_scalar(v.payload, v.dtype, (uint64_t)f));
        return fe_from_limbs<FrParams>(v.below[f].l);
    }
    TC_DEV void operator()(uint32_t lane) const {
        uint32_t h = lane & ((1u << logH) - 1u);
        uint32_t job = (lane >> logH) / terms_per_job, term = (lane >> logH) % terms_per_job;
        const NodeOpenJob& J = jobs[job];
        const LevelView& v = lv[J.level];
        int a = 0;
        while (a + 1 < node.m && term >= axis_first[a + 1]) ++a;
        uint32_t local = term - axis_first[a];
        /* child multi-index: axes < a fixed to kappa, axes >= a from `local` */
        uint32_t k[4];
        for (int j = 0; j < a; ++j) k[j] = J.kappa[j];
        unflatten(local, node, a, k);
        uint32_t kap = J.kappa[a], d = node.d[a];
        uint32_t kk[4];
        for (int j = 0; j < node.m; ++j) kk[j] = k[j];
        kk[a] = kap;
        fr_t gk = child_value(v, J.node, kk);
        fr_t qv;
        if (k[a] != kap) {
            uint32_t dist = k[a] > kap ? k[a] - kap : kap - k[a];
            qv = fr_mul(fr_sub(child_value(v, J.node, k), gk), ax[a].inv_int[dist]);
            if (k[a] < kap) qv = fr_neg(qv);
        } else {
            fr_t acc = fe_zero<FrParams>();
            for (uint32_t x = 0; x < d; ++x) {
                if (x == kap) continue;
                kk[a] = x;
                uint32_t dist = x > kap ? x - kap : kap - x;
                fr_t t = fr_mul(fr_sub(child_value(v, J.node, kk), gk), ax[a].inv_int[dist]);
                if (x < kap) t = fr_neg(t);
                acc = fr_add(acc, fr_mul(ax[a].beta[x], t));
            }
            qv = fr_neg(fr_mul(acc, ax[a].beta_inv[kap]));
        }
        fr_t plain = fe_to_plain(qv);
        out[(((uint64_t)J.term0 + term) << logH) + h] = fb_window_pair(table[a], local, plain.l, h);
        if (term == 0 && h == 0) {
            fr_t y = fe_to_plain(child_value(v, J.node, J.kappa));
#pragma unroll
            for (int i = 0; i < 8; ++i) y_out[job].l[i] = y.l[i];
        }
    }
};

/* ---- Ver (sum form, trapdoor-form check in G1) -------------------------------------------- */
/* One verification step: is  C - [y]G == sum_i [tau_i - (kappa_i + 1)] pi_i ?
 * Points arrive as canonical bytes; a point that is not on the curve rejects the step.
 * Each scalar k_i = tau_i - zeta_i arrives split as k_i = k1 + k2 lambda (both below 2^128), lambda the
 * eigenvalue of the endomorphism (x, y) -> (beta x, y), so that [k]P = [k1]P + [k2](beta x, y) costs two
 * half-length double-and-add chains that run in separate lanes. */
struct VerifyStep {
    uint32_t C[24];
    uint32_t y[8];
    uint32_t pi[4][24];
    uint32_t k1[4][4];
    uint32_t k2[4][4];
    int m;
};
constexpr uint32_t VERIFY_CHAINS = 8;     /* two half-scalar terms per proof element, at most four elements */
constexpr uint32_t VERIFY_BITS = 128;
TC_HD bool affine_on_curve(const g1_affine& p) {
    if (affine_is_identity(p)) return true;
    fp_t y2 = fp_sqr(p.y);
    fp_t x3 = fp_mul(fp_sqr(p.x), p.x);
    fp_t four = fe_from_u32<FpParams>(4);
    return fe_eq(y2, fp_add(x3, four));
}
TC_HD bool canonical_fp(const uint32_t* w) { return limbs_gt<12>(FpParams::MOD, w); }
TC_HD bool xyzz_equal(const g1_xyzz& a, const g1_xyzz& b) {
    bool ia = xyzz_is_identity(a), ib = xyzz_is_identity(b);
    if (ia || ib) return ia && ib;
    return fe_eq(fp_mul(a.X, b.ZZ), fp_mul(b.X, a.ZZ)) && fe_eq(fp_mul(a.Y, b.ZZZ), fp_mul(b.Y, a.ZZZ));
}
/* The 128 doublings of a half-length scalar multiplication cannot be spread over lanes, everything else can:
 * chain (step, j) of VerifyChain walks P, 2P, 4P, .. 2^127 P (chain 2i: P = pi_i, chain 2i + 1: its image
 * (beta x, y)) and keeps every point; cooperative sums then add, for a step, the points whose bit is set in
 * the half scalars, the window terms of [y]G and -C, and the step is accepted iff
 *   sum_i [k_i] pi_i + [y] G - C = O. */
/* Four waves per 64 chains.  The seven products of a Jacobian doubling (A = X^2, B = Y^2, Y Z; F = (3A)^2,
 * C = B^2, X B; E (D - X3)) fall into three levels of independent ones, and a wave alone on its SIMD issues them no
 * faster one after the other than three waves do side by side: wave 0 carries X and Y, wave 1 the powers of Y,
 * wave 2 Z and D = 4 X B; operands pass through LDS, a barrier after every level.  The chain computes in the
 * 28-bit-limb form of the field (a wave alone gets through those products 1.6 times as fast as through the 32-bit
 * ones: 0.81 -> 0.60 ms for the chains of eight paths): sums and small multiples are limb-wise and get one carry
 * pass before they meet a product, nothing is reduced along the way.  The points that the chain keeps are in the
 * 32-bit form; wave 3 converts them, one coordinate per level, from copies that the other waves leave for it (X
 * and Y of a point in the slot of its parity, so that the next doubling may write while the last is still being
 * read).  Z = 0 (the identity) reproduces itself under these formulas, so the loop has no special cases. */
struct VerifyChain {
    static constexpr int BLOCK = 256;
    enum { FX, FY, FZ, FE, FB, FC8, FD, FF, PZ, PX0, PX1, PY0, PY1, NFIELD };
    static constexpr size_t LDS_BYTES = (size_t)NFIELD * 4 * 64 * 16;
    static constexpr int PHASES = 1 + 3 * ((int)VERIFY_BITS - 1) + 2;
    struct Quad { int32_t v[4]; };
    const VerifyStep* steps;
    uint32_t n_chains;         /* VERIFY_CHAINS per step */
    uint32_t* ok;
    g1_jac* chain;

    TC_DEV static fp28 ld(const uint8_t* lds, int f, uint32_t l) {
        const Quad* q = (const Quad*)lds;
        fp28 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            Quad t = q[(f * 4 + i) * 64 + l];
            r.l[4 * i] = t.v[0]; r.l[4 * i + 1] = t.v[1];
            if (i < 3) { r.l[4 * i + 2] = t.v[2]; r.l[4 * i + 3] = t.v[3]; }
        }
        return r;
    }
    TC_DEV static void st(uint8_t* lds, int f, uint32_t l, const fp28& x) {
        Quad* q = (Quad*)lds;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            Quad t;
            t.v[0] = x.l[4 * i]; t.v[1] = x.l[4 * i + 1];
            t.v[2] = i < 3 ? x.l[4 * i + 2] : 0; t.v[3] = i < 3 ? x.l[4 * i + 3] : 0;
            q[(f * 4 + i) * 64 + l] = t;
        }
    }
    TC_DEV static fp28 times2(const fp28& a) { return fp28_add(a, a); }
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t* lds) const {
        uint32_t wave = lane >> 6, l = lane & 63u;
        uint32_t c = wg * 64u + l;
        bool live = false;
        if (c < n_chains) live = (int)((c % VERIFY_CHAINS) >> 1) < steps[c / VERIFY_CHAINS].m;
        g1_jac* out = chain + (uint64_t)c * VERIFY_BITS;
        if (ph == 0) {
            if (wave != 0) return;
            g1_jac q = jac_identity();
            if (live) {
                uint32_t s = c / VERIFY_CHAINS, j = c % VERIFY_CHAINS;
                const uint32_t* w = steps[s].pi[j >> 1];
                g1_affine p = affine_from_canonical(w);
                bool second = (j & 1u) != 0;
                if (!second && (!canonical_fp(w) || !canonical_fp(w + 12) || !affine_on_curve(p))) atomic_and_u32(&ok[s], 0u);
                if (!affine_is_identity(p)) {
                    if (second) {
                        fp_t beta;
#pragma unroll
                        for (int t = 0; t < 12; ++t) beta.l[t] = GLV_BETA[t];
                        p.x = fp_mul(p.x, beta);
                    }
                    q.X = p.x;
                    q.Y = p.y;
                    q.Z = fe_one<FpParams>();
                }
                out[0] = q;
            }
            st(lds, FX, l, fp28_from_fp(q.X));
            st(lds, FY, l, fp28_from_fp(q.Y));
            st(lds, FZ, l, fp28_from_fp(q.Z));
            return;
        }
        const int last = 1 + 3 * ((int)VERIFY_BITS - 1);
        if (ph >= last) {                       /* X and Y of the last point */
            if (wave != 3 || !live) return;
            const uint32_t b = VERIFY_BITS - 1;
            if (ph == last) out[b].X = fp28_to_fp(ld(lds, (b & 1u) ? PX1 : PX0, l));
            else out[b].Y = fp28_to_fp(ld(lds, (b & 1u) ? PY1 : PY0, l));
            return;
        }
        uint32_t b = (uint32_t)(ph - 1) / 3u + 1u;      /* the point 2^b P is in the making */
        int level = (ph - 1) % 3;
        if (wave == 3) {                        /* the converter: X of the point before, Z of this one, Y of the point before */
            if (!live) return;
            if (level == 0) {
                if (b > 1) out[b - 1].X = fp28_to_fp(ld(lds, ((b - 1) & 1u) ? PX1 : PX0, l));
            } else if (level == 1) {
                out[b].Z = fp28_to_fp(ld(lds, PZ, l));
            } else if (b > 1) {
                out[b - 1].Y = fp28_to_fp(ld(lds, ((b - 1) & 1u) ? PY1 : PY0, l));
            }
            return;
        }
        if (level == 0) {
            if (wave == 0) {
                fp28 A = fp28_sqr(ld(lds, FX, l));
                st(lds, FE, l, fp28_carry(fp28_add(times2(A), A)));
            } else if (wave == 1) {
                st(lds, FB, l, fp28_sqr(ld(lds, FY, l)));
            } else {
                fp28 Z3 = times2(fp28_mul(ld(lds, FY, l), ld(lds, FZ, l)));       /* limbs below 2^29: a factor of the next Y Z only */
                st(lds, FZ, l, Z3);
                st(lds, PZ, l, Z3);
            }
            return;
        }
        if (level == 1) {
            if (wave == 0) {
                st(lds, FF, l, fp28_sqr(ld(lds, FE, l)));
            } else if (wave == 1) {
                fp28 C = fp28_sqr(ld(lds, FB, l));
                st(lds, FC8, l, fp28_carry(times2(times2(times2(C)))));
            } else {
                fp28 XB = fp28_mul(ld(lds, FX, l), ld(lds, FB, l));
                st(lds, FD, l, fp28_carry(times2(times2(XB))));
            }
            return;
        }
        if (wave == 0) {
            fp28 D = ld(lds, FD, l);
            fp28 X3 = fp28_carry(fp28_sub(fp28_sub(ld(lds, FF, l), D), D));
            fp28 Y3 = fp28_carry(fp28_sub(fp28_mul(ld(lds, FE, l), fp28_sub(D, X3)), ld(lds, FC8, l)));
            st(lds, FX, l, X3);
            st(lds, FY, l, Y3);
            st(lds, (b & 1u) ? PX1 : PX0, l, X3);
            st(lds, (b & 1u) ? PY1 : PY0, l, Y3);
        }
    }
};
/* What the cooperative sums of a step add: group g < groups - 1 the points of chains 2g and 2g + 1 whose bit is
 * set (an identity elsewhere), the last group the window terms of [y]G and -C; `groups` is one more than the
 * largest order among the steps of the launch. */
struct VerifyGroupSrc {
    const VerifyStep* steps;
    const g1_affine* gtable;
    const g1_jac* chain;
    uint32_t* ok;
    uint32_t groups;
    g1_xyzz* partial;          /* steps * groups */
    TC_DEV uint32_t count(uint32_t wg) const {
        uint32_t s = wg / groups, g = wg % groups;
        if (g + 1 == groups) return (uint32_t)FB_W + 1u;
        return (int)g < steps[s].m ? 2u * VERIFY_BITS : 0u;
    }
    TC_DEV g1_xyzz load(uint32_t wg, uint32_t i) const {
        uint32_t s = wg / groups, g = wg % groups;
        const VerifyStep& st = steps[s];
        if (g + 1 < groups) {
            uint32_t j = 2 * g + i / VERIFY_BITS, b = i % VERIFY_BITS;
            const uint32_t* k = (j & 1u) ? st.k2[j >> 1] : st.k1[j >> 1];
            if (!((k[b >> 5] >> (b & 31)) & 1u)) return xyzz_identity();
            return jac_to_xyzz(chain[((uint64_t)s * VERIFY_CHAINS + j) * VERIFY_BITS + b]);
        }
        g1_affine p = affine_identity();
        if (i < (uint32_t)FB_W) {                /* window i of [y] G */
            uint32_t carry = 0;
            int32_t d = 0;
            for (uint32_t w = 0; w <= i; ++w) d = fr_window_digit(st.y, (int)w, FB_C, carry);
            if (d) {
                p = gtable[(uint64_t)i * FB_NB + (uint32_t)(d < 0 ? -d : d) - 1u];
                if (d < 0) p.y = fp_neg(p.y);
            }
        } else {                                 /* -C, and the checks on C and y */
            p = affine_from_canonical(st.C);
            bool good = canonical_fp(st.C) && canonical_fp(st.C + 12) && affine_on_curve(p) && limbs_gt<8>(FrParams::MOD, st.y);
            if (!good) atomic_and_u32(&ok[s], 0u);
            p = affine_neg(p);
        }
        return xyzz_from_affine(p);
    }
    TC_DEV void store(uint32_t wg, const g1_xyzz& r) const { partial[wg] = r; }
};
struct VerifyDecideSrc {       /* workgroup = step: the partial sums must cancel */
    const g1_xyzz* partial;
    uint32_t groups;
    uint32_t* ok;
    TC_DEV uint32_t count(uint32_t) const { return groups; }
    TC_DEV g1_xyzz load(uint32_t s, uint32_t i) const { return partial[(uint64_t)s * groups + i]; }
    TC_DEV void store(uint32_t s, const g1_xyzz& r) const {
        if (!xyzz_is_identity(r)) ok[s] = 0;
    }
};
constexpr uint32_t VERIFY_MAX_GROUPS = VERIFY_CHAINS / 2 + 1;
/* canonical bytes -> affine point in Montgomery form; a point that is not canonical or not on the curve clears *ok */
struct FromCanonicalChecked {
    const uint32_t* in;     /* 24 words per point */
    g1_affine* out;
    uint32_t* ok;
    TC_DEV void operator()(uint32_t t) const {
        const uint32_t* w = in + 24 * (uint64_t)t;
        g1_affine p = affine_from_canonical(w);
        if (!limbs_gt<12>(FpParams::MOD, w) || !limbs_gt<12>(FpParams::MOD, w + 12) || !affine_on_curve(p)) atomic_and_u32(ok, 0u);
        out[t] = p;
    }
};
/* phi of canonical commitments (the verifier's side of "the opened value matches the next commitment") */
struct PhiCanonical {
    const uint32_t* pts;       /* 24 words each */
    fr_plain* out;
    TC_DEV void operator()(uint32_t t) const {
        fr_t v = phi_map(affine_from_canonical(pts + 24 * (uint64_t)t));
#pragma unroll
        for (int i = 0; i < 8; ++i) out[t].l[i] = v.l[i];
    }
};

/* ---- the coefficient route: interpolation along one axis, Algorithm 1 ------------------------ */
/* Lines of length d along one axis of an (outer, d, inner) array of Montgomery Fr values, nodes zeta_k = k + 1.
 * A workgroup owns `lines_per_wg` whole lines; a barrier separates the phases, values move between three
 * arrays in global memory (buf[0] holds the input):
 *   phases 0 .. d-2       divided differences, level l = phase + 1:  c_k <- (c_k - c_(k-1)) / l  for k >= l
 *                         (equispaced nodes: zeta_k - zeta_(k-l) = l), ping-pong between buf[0] and buf[1];
 *   phase d-1             a = (c_(d-1), 0, .., 0)
 *   phases d .. 2d-2      step s = phase - (d-1), k = d-1-s:  a <- a (x - zeta_k) + c_k, i.e.
 *                         a_i <- a_(i-1) - zeta_k a_i (+ c_k at i = 0), ping-pong between the two arrays
 *                         that do not hold c.
 * The host works out where c and the result end up (interp_result_buffer).
 * Gregory form (a second instantiation, so that the Newton kernel keeps its register count and with it two
 * workgroups per CU): the levels take plain forward differences, c_k <- c_k - c_(k-1), so that
 * c_k = Delta^k T[0], and the expansion reads c_k / k!, the coefficient of N_k in
 * sum_k binom(X - zeta_0, k) Delta^k T[0] (h = 1). */
template <bool GREGORY>
struct InterpAxis {
    static constexpr int BLOCK = 1024;       /* a long line is bound by its 2d - 1 barriers: as many lanes as a workgroup has */
    static constexpr size_t LDS_BYTES = 16;
    fr_t* buf[3];
    uint64_t outer, inner;
    uint32_t d, lines_per_wg;
    const fr_t* inv_int;       /* inv_int[l] = 1 / l, l = 1 .. d-1 */
    const fr_t* zeta;          /* zeta[k] = k + 1 */
    const fr_t* inv_fact;      /* Gregory form only: inv_fact[l] = 1 / l! */
    TC_DEV fr_t newton_coefficient(const fr_t* c, uint64_t base, uint32_t k) const {
        fr_t v = c[base + (uint64_t)k * inner];
        return GREGORY ? fr_mul(v, inv_fact[k]) : v;
    }
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t*) const {
        uint64_t lines = outer * inner;
        int cbuf = (int)((d - 1) & 1u);                  /* c after the d - 1 levels */
        int pa = cbuf == 0 ? 1 : 0, pb = 2;              /* the two arrays of the expansion */
        for (uint64_t idx = lane; idx < (uint64_t)lines_per_wg * d; idx += BLOCK) {
            uint64_t line = (uint64_t)wg * lines_per_wg + idx / d;
            uint32_t k = (uint32_t)(idx % d);
            if (line >= lines) continue;
            uint64_t base = (line / inner) * d * inner + line % inner;
            uint64_t at = base + (uint64_t)k * inner;
            if (ph + 1 < (int)d) {
                uint32_t l = (uint32_t)ph + 1;
                const fr_t* src = buf[ph & 1];
                fr_t v = src[at];
                if (k >= l) {
                    v = fr_sub(v, src[at - inner]);
                    if (!GREGORY) v = fr_mul(v, inv_int[l]);
                }
                buf[(ph + 1) & 1][at] = v;
            } else if (ph + 1 == (int)d) {
                buf[pa][at] = k == 0 ? newton_coefficient(buf[cbuf], base, d - 1) : fe_zero<FrParams>();
            } else {
                uint32_t s = (uint32_t)ph - (d - 1), kk = d - 1 - s;
                const fr_t* old = buf[(s & 1u) ? pa : pb];
                fr_t* nxt = buf[(s & 1u) ? pb : pa];
                fr_t v = fr_neg(fr_mul(zeta[kk], old[at]));
                v = fr_add(v, k ? old[at - inner] : newton_coefficient(buf[cbuf], base, kk));
                nxt[at] = v;
            }
        }
    }
};
/* index (0..2) of the array that holds the coefficients after all 2d - 1 phases */
TC_HD int interp_result_buffer(uint32_t d) {
    int cbuf = (int)((d - 1) & 1u);
    int pa = cbuf == 0 ? 1 : 0, pb = 2;
    return ((d - 1) & 1u) ? pb : pa;
}
/* Barycentric form (App. C) of the same interpolation: f(X) = sum_l w_l prod_(r != l) (X - zeta_r) with
 * w_l = beta_l T_l.  Built node by node: with M_n = prod_(r < n) (X - zeta_r) and P_n the sum restricted to the
 * first n nodes, P_(n+1) = (X - zeta_n) P_n + w_n M_n and M_(n+1) = (X - zeta_n) M_n.  Lane = coefficient k of a
 * line; phase 0 forms w (in place) and sets P_0 = 0, M_0 = 1; phase n + 1 takes step n, P and M each moving
 * between two arrays.  After d steps the coefficients are in p[d & 1]. */
struct InterpAxisBarycentric {
    static constexpr int BLOCK = 1024;
    static constexpr size_t LDS_BYTES = 16;
    fr_t* w;                   /* the values on entry */
    fr_t* p[2];
    fr_t* mm[2];
    uint64_t outer, inner;
    uint32_t d, lines_per_wg;
    const fr_t* beta;          /* beta[l] = 1 / prod_(r != l) (zeta_l - zeta_r) */
    const fr_t* zeta;          /* zeta[k] = k + 1 */
    TC_DEV void phase(int ph, uint32_t lane, uint32_t wg, uint8_t*) const {
        uint64_t lines = outer * inner;
        for (uint64_t idx = lane; idx < (uint64_t)lines_per_wg * d; idx += BLOCK) {
            uint64_t line = (uint64_t)wg * lines_per_wg + idx / d;
            uint32_t k = (uint32_t)(idx % d);
            if (line >= lines) continue;
            uint64_t base = (line / inner) * d * inner + line % inner;
            uint64_t at = base + (uint64_t)k * inner;
            if (ph == 0) {
                w[at] = fr_mul(w[at], beta[k]);
                p[0][at] = fe_zero<FrParams>();
                mm[0][at] = k == 0 ? fe_one<FrParams>() : fe_zero<FrParams>();
                continue;
            }
            uint32_t n = (uint32_t)ph - 1;
            const fr_t* po = p[n & 1u];
            const fr_t* mo = mm[n & 1u];
            fr_t m_here = mo[at];
            fr_t pv = fr_add(fr_neg(fr_mul(zeta[n], po[at])), fr_mul(w[base + (uint64_t)n * inner], m_here));
            fr_t mv = fr_neg(fr_mul(zeta[n], m_here));
            if (k) {
                pv = fr_add(pv, po[at - inner]);
                mv = fr_add(mv, mo[at - inner]);
            }
            p[(n + 1) & 1u][at] = pv;
            mm[(n + 1) & 1u][at] = mv;
        }
    }
};
struct ScalarsToFr {           /* any scalar type -> Montgomery Fr */
    const void* scalars;
    int dtype;
    fr_t* out;
    TC_DEV void operator()(uint32_t t) const { out[t] = scalar_as_fr(scalars, dtype, t); }
};
struct FrToPlain {             /* Montgomery -> canonical 32 bytes */
    const fr_t* in;
    fr_plain* out;
    TC_DEV void operator()(uint32_t t) const {
        fr_t v = fe_to_plain(in[t]);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[t].l[i] = v.l[i];
    }
};
/* Algorithm 1 along one axis (App. A): lane = line; from the top degree down, the coefficient at degree c goes to
 * degree c - 1 of the quotient and, times omega, into degree c - 1 of the remainder. */
struct DivideAxis {
    const fr_plain* coeffs;
    uint64_t outer, inner;
    uint32_t d;
    uint32_t omega;
    fr_plain* q;
    fr_plain* r;
    TC_DEV void operator()(uint32_t t) const {
        uint64_t base = ((uint64_t)t / inner) * d * inner + (uint64_t)t % inner;
        fr_t w = fe_from_u32<FrParams>(omega);
        fr_t carry = fe_from_limbs<FrParams>(coeffs[base + (uint64_t)(d - 1) * inner].l);
        fr_plain zero;
#pragma unroll
        for (int i = 0; i < 8; ++i) zero.l[i] = 0;
        q[base + (uint64_t)(d - 1) * inner] = zero;
        for (uint32_t c = d - 1; c >= 1; --c) {
            fr_t plain = fe_to_plain(carry);
            fr_plain o;
#pragma unroll
            for (int i = 0; i < 8; ++i) o.l[i] = plain.l[i];
            q[base + (uint64_t)(c - 1) * inner] = o;
            r[base + (uint64_t)c * inner] = zero;
            carry = fr_add(fe_from_limbs<FrParams>(coeffs[base + (uint64_t)(c - 1) * inner].l), fr_mul(w, carry));
        }
        fr_t plain = fe_to_plain(carry);
        fr_plain o;
#pragma unroll
        for (int i = 0; i < 8; ++i) o.l[i] = plain.l[i];
        r[base] = o;
    }
};

/* ---- incremental update of one path (the structure is reused, Sec. 4.2) ---------------------- */
/* The commitment of node `a` of a level moves by [s] B, where B is base `k` of a fixed-base table (nodes) or one
 * SRS point (a leaf tensor) and s is a small signed integer (an entry changed) or the change of phi of the child
 * below (read from `dphi`, written by the launch for the level below).  A cooperative sum adds the old
 * commitment and the window terms of [s] B; its last lane standing normalises, replaces the commitment and its
 * phi, and leaves the change of phi in `dphi` for the level above. */
struct UpdatePathSrc {
    g1_affine* C;              /* level array */
    fr_plain* phi;
    uint64_t a;
    const g1_affine* table;    /* fixed-base table, or null */
    uint32_t k;
    const g1_affine* point;    /* single base when table is null */
    int64_t small;             /* used when from_dphi == 0 */
    int from_dphi;
    fr_plain* dphi;            /* one value */
    TC_DEV fr_t scalar() const {
        if (from_dphi) return fe_from_limbs<FrParams>(dphi->l);
        uint64_t mag = (uint64_t)(small < 0 ? -small : small);
        uint32_t w[8] = {(uint32_t)mag, (uint32_t)(mag >> 32), 0, 0, 0, 0, 0, 0};
        fr_t s = fe_from_limbs<FrParams>(w);
        return small < 0 ? fr_neg(s) : s;
    }
    TC_DEV uint32_t count(uint32_t) const { return table ? (uint32_t)FB_W + 1u : 2u; }
    TC_DEV g1_xyzz load(uint32_t, uint32_t i) const {
        if (i == 0) return xyzz_from_affine(C[a]);
        fr_t plain = fe_to_plain(scalar());
        if (!table) return xyzz_mul_affine(plain.l, 256, *point);
        uint32_t w = i - 1, carry = 0;
        int32_t d = 0;
        for (uint32_t x = 0; x <= w; ++x) d = fr_window_digit(plain.l, (int)x, FB_C, carry);
        if (!d) return xyzz_identity();
        g1_affine p = table[((uint64_t)k * FB_W + w) * FB_NB + (uint32_t)(d < 0 ? -d : d) - 1u];
        if (d < 0) p.y = fp_neg(p.y);
        return xyzz_from_affine(p);
    }
    TC_DEV void store(uint32_t, const g1_xyzz& r) const {
        g1_affine c = xyzz_to_affine(r);
        fr_t old_phi = fe_from_limbs<FrParams>(phi[a].l);
        fr_t new_plain = phi_map(c);
        fr_t diff = fe_to_plain(fr_sub(fe_from_limbs<FrParams>(new_plain.l), old_phi));
        C[a] = c;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            phi[a].l[i] = new_plain.l[i];
            dphi->l[i] = diff.l[i];
        }
    }
};

}  // namespace tc
