/*
 * Plain-C oracle for the TensorCommitments prover path.  TEST INFRASTRUCTURE ONLY.
 *
 * It exists so that the oracle can reach sizes Python integers cannot reach in
 * seconds, and so that the CPU baseline is timed on compiled code.  It shares
 * no code with the HIP library.  What it computes:
 *
 *   - Fr / Fp arithmetic on 64-bit limbs: schoolbook product to double width,
 *     then reduction by folding the high limbs through the table
 *     2^(64 k) mod q (a congruence, nothing else), then subtracting q while
 *     the value is >= q.  No Montgomery form, no Barrett.
 *   - G1 of BLS12-381 (the curve App. E names) in Jacobian coordinates with
 *     the textbook formulas and explicit identity / equal / opposite cases.
 *   - Com_TC of Def. 4.1 as the multi-exponentiation written out term by
 *     term: every term its own MSB-first double-and-add (no windows, no
 *     buckets), partial sums per thread, one inversion at the end.
 *   - f_T(tau) = sum_i T[i] prod_j l_{j,i_j}(tau_j): nested sums, last axis
 *     first (the closed form of Def. 4.1 under a known trapdoor).
 *
 * Encodings: Fr = 32 bytes little-endian (< r); G1 = x || y, 48 bytes
 * little-endian each, affine; identity = 96 zero bytes.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef unsigned __int128 u128;

#define FR_N 4
#define FP_N 6
#define MAXN 6

typedef struct {
    int n;                       /* limbs */
    uint64_t q[MAXN];            /* modulus */
    uint64_t fold[MAXN + 1][MAXN]; /* fold[k] = 2^(64 (n + k)) mod q, k = 0..n */
} modulus_t;

static modulus_t FR, FP;
static int g_ready = 0;

/* ---- multi-limb helpers ---------------------------------------------------- */
static int ge(const uint64_t* a, const uint64_t* b, int n) {
    for (int i = n - 1; i >= 0; --i) {
        if (a[i] > b[i]) return 1;
        if (a[i] < b[i]) return 0;
    }
    return 1;
}
static uint64_t add_n(uint64_t* r, const uint64_t* a, const uint64_t* b, int n) {
    u128 c = 0;
    for (int i = 0; i < n; ++i) {
        c += (u128)a[i] + b[i];
        r[i] = (uint64_t)c;
        c >>= 64;
    }
    return (uint64_t)c;
}
static uint64_t sub_n(uint64_t* r, const uint64_t* a, const uint64_t* b, int n) {
    uint64_t borrow = 0;
    for (int i = 0; i < n; ++i) {
        u128 d = (u128)a[i] - b[i] - borrow;
        r[i] = (uint64_t)d;
        borrow = (uint64_t)(d >> 64) & 1;
    }
    return borrow;
}
static int is_zero(const uint64_t* a, int n) {
    uint64_t o = 0;
    for (int i = 0; i < n; ++i) o |= a[i];
    return o == 0;
}

static void mod_add(const modulus_t* M, uint64_t* r, const uint64_t* a, const uint64_t* b) {
    uint64_t t[MAXN];
    uint64_t carry = add_n(t, a, b, M->n);
    if (carry || ge(t, M->q, M->n)) sub_n(t, t, M->q, M->n);
    memcpy(r, t, sizeof(uint64_t) * M->n);
}
static void mod_sub(const modulus_t* M, uint64_t* r, const uint64_t* a, const uint64_t* b) {
    uint64_t t[MAXN];
    if (sub_n(t, a, b, M->n)) add_n(t, t, M->q, M->n);
    memcpy(r, t, sizeof(uint64_t) * M->n);
}
static void mod_neg(const modulus_t* M, uint64_t* r, const uint64_t* a) {
    uint64_t z[MAXN] = {0};
    mod_sub(M, r, z, a);
}

/* value (len limbs, len <= 2n+1) -> value mod q in r[0..n) */
static void mod_reduce(const modulus_t* M, uint64_t* r, const uint64_t* x, int len) {
    int n = M->n;
    uint64_t cur[2 * MAXN + 2];
    memset(cur, 0, sizeof cur);
    memcpy(cur, x, sizeof(uint64_t) * len);
    for (;;) {
        int top = 0;
        for (int i = n; i < 2 * MAXN + 2; ++i) if (cur[i]) top = 1;
        if (!top) break;
        /* acc = low n limbs + sum_k cur[n + k] * fold[k] */
        uint64_t acc[2 * MAXN + 2];
        memset(acc, 0, sizeof acc);
        memcpy(acc, cur, sizeof(uint64_t) * n);
        for (int k = 0; k <= n && n + k < 2 * MAXN + 2; ++k) {
            uint64_t h = cur[n + k];
            if (!h) continue;
            u128 c = 0;
            int i;
            for (i = 0; i < n; ++i) {
                c += (u128)h * M->fold[k][i] + acc[i];
                acc[i] = (uint64_t)c;
                c >>= 64;
            }
            for (; c && i < 2 * MAXN + 2; ++i) {
                c += acc[i];
                acc[i] = (uint64_t)c;
                c >>= 64;
            }
        }
        memcpy(cur, acc, sizeof cur);
    }
    while (ge(cur, M->q, n)) sub_n(cur, cur, M->q, n);
    memcpy(r, cur, sizeof(uint64_t) * n);
}

static void mod_mul(const modulus_t* M, uint64_t* r, const uint64_t* a, const uint64_t* b) {
    int n = M->n;
    uint64_t t[2 * MAXN];
    memset(t, 0, sizeof t);
    for (int i = 0; i < n; ++i) {               /* schoolbook product */
        u128 c = 0;
        for (int j = 0; j < n; ++j) {
            c += (u128)a[i] * b[j] + t[i + j];
            t[i + j] = (uint64_t)c;
            c >>= 64;
        }
        t[i + n] = (uint64_t)c;
    }
    mod_reduce(M, r, t, 2 * n);
}

/* a^e, e given as n limbs (square and multiply, MSB first) */
static void mod_pow(const modulus_t* M, uint64_t* r, const uint64_t* a, const uint64_t* e) {
    uint64_t acc[MAXN] = {1};
    for (int i = M->n * 64 - 1; i >= 0; --i) {
        mod_mul(M, acc, acc, acc);
        if ((e[i / 64] >> (i % 64)) & 1) mod_mul(M, acc, acc, a);
    }
    memcpy(r, acc, sizeof(uint64_t) * M->n);
}
static void mod_inv(const modulus_t* M, uint64_t* r, const uint64_t* a) {   /* Fermat */
    uint64_t e[MAXN], two[MAXN] = {2};
    sub_n(e, M->q, two, M->n);
    mod_pow(M, r, a, e);
}

static void modulus_init(modulus_t* M, int n, const uint64_t* q) {
    M->n = n;
    memcpy(M->q, q, sizeof(uint64_t) * n);
    /* 2^(64 n) mod q by 64 n doublings of 1, then 64 more per further table row */
    uint64_t v[MAXN] = {1};
    for (int k = 0; k <= n; ++k) {
        int steps = (k == 0) ? 64 * n : 64;
        for (int s = 0; s < steps; ++s) mod_add(M, v, v, v);
        memcpy(M->fold[k], v, sizeof(uint64_t) * n);
    }
}

static void from_le(uint64_t* r, const uint8_t* b, int n) {
    for (int i = 0; i < n; ++i) {
        uint64_t w = 0;
        for (int k = 7; k >= 0; --k) w = (w << 8) | b[8 * i + k];
        r[i] = w;
    }
}
static void to_le(uint8_t* b, const uint64_t* a, int n) {
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < 8; ++k) b[8 * i + k] = (uint8_t)(a[i] >> (8 * k));
}

/* ---- G1, Jacobian ----------------------------------------------------------- */
typedef struct { uint64_t X[FP_N], Y[FP_N], Z[FP_N]; } jac_t;   /* Z == 0: identity */

static uint64_t G1X[FP_N], G1Y[FP_N];

static void jac_set_inf(jac_t* p) { memset(p, 0, sizeof *p); p->X[0] = 1; p->Y[0] = 1; }
static int jac_is_inf(const jac_t* p) { return is_zero(p->Z, FP_N); }

static void jac_double(jac_t* r, const jac_t* a) {
    if (jac_is_inf(a) || is_zero(a->Y, FP_N)) { jac_set_inf(r); return; }
    uint64_t A[FP_N], B[FP_N], C[FP_N], D[FP_N], E[FP_N], F[FP_N], t[FP_N], X3[FP_N], Y3[FP_N], Z3[FP_N];
    mod_mul(&FP, A, a->X, a->X);
    mod_mul(&FP, B, a->Y, a->Y);
    mod_mul(&FP, C, B, B);
    mod_add(&FP, t, a->X, B);
    mod_mul(&FP, t, t, t);
    mod_sub(&FP, t, t, A);
    mod_sub(&FP, t, t, C);
    mod_add(&FP, D, t, t);                 /* D = 2((X+B)^2 - A - C) */
    mod_add(&FP, E, A, A);
    mod_add(&FP, E, E, A);                 /* E = 3A */
    mod_mul(&FP, F, E, E);
    mod_sub(&FP, X3, F, D);
    mod_sub(&FP, X3, X3, D);               /* X3 = F - 2D */
    mod_sub(&FP, t, D, X3);
    mod_mul(&FP, Y3, E, t);
    mod_add(&FP, C, C, C);
    mod_add(&FP, C, C, C);
    mod_add(&FP, C, C, C);                 /* 8C */
    mod_sub(&FP, Y3, Y3, C);
    mod_mul(&FP, Z3, a->Y, a->Z);
    mod_add(&FP, Z3, Z3, Z3);
    memcpy(r->X, X3, sizeof X3); memcpy(r->Y, Y3, sizeof Y3); memcpy(r->Z, Z3, sizeof Z3);
}

static void jac_add(jac_t* r, const jac_t* a, const jac_t* b) {
    if (jac_is_inf(a)) { *r = *b; return; }
    if (jac_is_inf(b)) { *r = *a; return; }
    uint64_t Z1Z1[FP_N], Z2Z2[FP_N], U1[FP_N], U2[FP_N], S1[FP_N], S2[FP_N], H[FP_N], Rr[FP_N];
    mod_mul(&FP, Z1Z1, a->Z, a->Z);
    mod_mul(&FP, Z2Z2, b->Z, b->Z);
    mod_mul(&FP, U1, a->X, Z2Z2);
    mod_mul(&FP, U2, b->X, Z1Z1);
    mod_mul(&FP, S1, a->Y, b->Z); mod_mul(&FP, S1, S1, Z2Z2);
    mod_mul(&FP, S2, b->Y, a->Z); mod_mul(&FP, S2, S2, Z1Z1);
    mod_sub(&FP, H, U2, U1);
    mod_sub(&FP, Rr, S2, S1);
    if (is_zero(H, FP_N)) {
        if (is_zero(Rr, FP_N)) jac_double(r, a); else jac_set_inf(r);
        return;
    }
    uint64_t HH[FP_N], HHH[FP_N], V[FP_N], X3[FP_N], Y3[FP_N], Z3[FP_N], t[FP_N];
    mod_mul(&FP, HH, H, H);
    mod_mul(&FP, HHH, H, HH);
    mod_mul(&FP, V, U1, HH);
    mod_mul(&FP, X3, Rr, Rr);
    mod_sub(&FP, X3, X3, HHH);
    mod_sub(&FP, X3, X3, V);
    mod_sub(&FP, X3, X3, V);               /* X3 = R^2 - H^3 - 2V */
    mod_sub(&FP, t, V, X3);
    mod_mul(&FP, Y3, Rr, t);
    mod_mul(&FP, t, S1, HHH);
    mod_sub(&FP, Y3, Y3, t);               /* Y3 = R(V - X3) - S1 H^3 */
    mod_mul(&FP, Z3, H, a->Z);
    mod_mul(&FP, Z3, Z3, b->Z);
    memcpy(r->X, X3, sizeof X3); memcpy(r->Y, Y3, sizeof Y3); memcpy(r->Z, Z3, sizeof Z3);
}

static void jac_from_bytes(jac_t* p, const uint8_t* b) {
    int zero = 1;
    for (int i = 0; i < 96; ++i) if (b[i]) zero = 0;
    if (zero) { jac_set_inf(p); return; }
    from_le(p->X, b, FP_N);
    from_le(p->Y, b + 48, FP_N);
    memset(p->Z, 0, sizeof p->Z);
    p->Z[0] = 1;
}
static void jac_to_bytes(uint8_t* b, const jac_t* p) {
    if (jac_is_inf(p)) { memset(b, 0, 96); return; }
    uint64_t zi[FP_N], zi2[FP_N], x[FP_N], y[FP_N];
    mod_inv(&FP, zi, p->Z);
    mod_mul(&FP, zi2, zi, zi);
    mod_mul(&FP, x, p->X, zi2);
    mod_mul(&FP, y, p->Y, zi2);
    mod_mul(&FP, y, y, zi);
    to_le(b, x, FP_N);
    to_le(b + 48, y, FP_N);
}
static void jac_neg(jac_t* p) { if (!jac_is_inf(p)) mod_neg(&FP, p->Y, p->Y); }

/* [k]P, k as `bits`-bit little-endian limbs, MSB-first double-and-add */
static void jac_mul(jac_t* r, const uint64_t* k, int nlimbs, const jac_t* P) {
    jac_t acc;
    jac_set_inf(&acc);
    for (int i = nlimbs * 64 - 1; i >= 0; --i) {
        jac_double(&acc, &acc);
        if ((k[i / 64] >> (i % 64)) & 1) jac_add(&acc, &acc, P);
    }
    *r = acc;
}

/* ---- exported ---------------------------------------------------------------- */
int tco_init(void) {
    if (g_ready) return 0;
    static const uint64_t r_[FR_N] = {0xffffffff00000001ULL, 0x53bda402fffe5bfeULL, 0x3339d80809a1d805ULL,
                                      0x73eda753299d7d48ULL};
    static const uint64_t p_[FP_N] = {0xb9feffffffffaaabULL, 0x1eabfffeb153ffffULL, 0x6730d2a0f6b0f624ULL,
                                      0x64774b84f38512bfULL, 0x4b1ba7b6434bacd7ULL, 0x1a0111ea397fe69aULL};
    static const uint64_t gx[FP_N] = {0xfb3af00adb22c6bbULL, 0x6c55e83ff97a1aefULL, 0xa14e3a3f171bac58ULL,
                                      0xc3688c4f9774b905ULL, 0x2695638c4fa9ac0fULL, 0x17f1d3a73197d794ULL};
    static const uint64_t gy[FP_N] = {0x0caa232946c5e7e1ULL, 0xd03cc744a2888ae4ULL, 0x00db18cb2c04b3edULL,
                                      0xfcf5e095d5d00af6ULL, 0xa09e30ed741d8ae4ULL, 0x08b3f481e3aaa0f1ULL};
    modulus_init(&FR, FR_N, r_);
    modulus_init(&FP, FP_N, p_);
    memcpy(G1X, gx, sizeof gx);
    memcpy(G1Y, gy, sizeof gy);
    g_ready = 1;
    return 0;
}

void tco_fr_mul(const uint8_t a[32], const uint8_t b[32], uint8_t out[32]) {
    uint64_t x[FR_N], y[FR_N];
    tco_init();
    from_le(x, a, FR_N); from_le(y, b, FR_N);
    mod_mul(&FR, x, x, y);
    to_le(out, x, FR_N);
}
void tco_fp_mul(const uint8_t a[48], const uint8_t b[48], uint8_t out[48]) {
    uint64_t x[FP_N], y[FP_N];
    tco_init();
    from_le(x, a, FP_N); from_le(y, b, FP_N);
    mod_mul(&FP, x, x, y);
    to_le(out, x, FP_N);
}
void tco_fp_inv(const uint8_t a[48], uint8_t out[48]) {
    uint64_t x[FP_N];
    tco_init();
    from_le(x, a, FP_N);
    mod_inv(&FP, x, x);
    to_le(out, x, FP_N);
}
void tco_g1_add(const uint8_t a[96], const uint8_t b[96], uint8_t out[96]) {
    jac_t x, y;
    tco_init();
    jac_from_bytes(&x, a); jac_from_bytes(&y, b);
    jac_add(&x, &x, &y);
    jac_to_bytes(out, &x);
}
void tco_g1_mul(const uint8_t k[32], const uint8_t pt[96], uint8_t out[96]) {
    jac_t x;
    uint64_t s[FR_N];
    tco_init();
    from_le(s, k, FR_N);
    jac_from_bytes(&x, pt);
    jac_mul(&x, s, FR_N, &x);
    jac_to_bytes(out, &x);
}
void tco_g1_generator(uint8_t out[96]) {
    tco_init();
    to_le(out, G1X, FP_N);
    to_le(out + 48, G1Y, FP_N);
}

/* scalar kinds */
enum { TCO_I8 = 1, TCO_I16 = 2, TCO_FR = 3 };

typedef struct {
    const void* scalars; int kind; const uint8_t* points; size_t lo, hi; jac_t sum;
} msm_job_t;

static void* msm_worker(void* arg) {
    msm_job_t* j = (msm_job_t*)arg;
    jac_t acc, term, base;
    jac_set_inf(&acc);
    for (size_t i = j->lo; i < j->hi; ++i) {
        jac_from_bytes(&base, j->points + 96 * i);
        if (j->kind == TCO_FR) {
            uint64_t s[FR_N];
            from_le(s, (const uint8_t*)j->scalars + 32 * i, FR_N);
            jac_mul(&term, s, FR_N, &base);
        } else {
            /* e(q) = r - |q| for q < 0, and [r - |q|]P = -[|q|]P */
            int64_t q = (j->kind == TCO_I8) ? ((const int8_t*)j->scalars)[i] : ((const int16_t*)j->scalars)[i];
            uint64_t mag = (uint64_t)(q < 0 ? -q : q);
            jac_mul(&term, &mag, 1, &base);
            if (q < 0) jac_neg(&term);
        }
        jac_add(&acc, &acc, &term);
    }
    j->sum = acc;
    return 0;
}

/* C = sum_i [e(s_i)] P_i, every term by its own double-and-add; returns threads used */
int tco_msm_naive(const void* scalars, int kind, const uint8_t* points, size_t n, int nthreads, uint8_t out[96]) {
    tco_init();
    if (nthreads < 1) nthreads = 1;
    if ((size_t)nthreads > n) nthreads = n ? (int)n : 1;
    msm_job_t* jobs = (msm_job_t*)calloc(nthreads, sizeof *jobs);
    pthread_t* th = (pthread_t*)calloc(nthreads, sizeof *th);
    for (int t = 0; t < nthreads; ++t) {
        jobs[t].scalars = scalars; jobs[t].kind = kind; jobs[t].points = points;
        jobs[t].lo = n * t / nthreads; jobs[t].hi = n * (t + 1) / nthreads;
        pthread_create(&th[t], 0, msm_worker, &jobs[t]);
    }
    jac_t acc;
    jac_set_inf(&acc);
    for (int t = 0; t < nthreads; ++t) {
        pthread_join(th[t], 0);
        jac_add(&acc, &acc, &jobs[t].sum);
    }
    jac_to_bytes(out, &acc);
    free(jobs); free(th);
    return nthreads;
}

/* one contraction of the last axis: out[o] = sum_k e(v[o*d + k]) * ell[k] mod r */
typedef struct { const void* v; int kind; size_t d; const uint64_t* ell; size_t lo, hi; uint8_t* out; } ctr_job_t;

static void* ctr_worker(void* arg) {
    ctr_job_t* j = (ctr_job_t*)arg;
    for (size_t o = j->lo; o < j->hi; ++o) {
        uint64_t acc[FR_N] = {0}, x[FR_N], t[FR_N];
        for (size_t k = 0; k < j->d; ++k) {
            size_t i = o * j->d + k;
            if (j->kind == TCO_FR) {
                from_le(x, (const uint8_t*)j->v + 32 * i, FR_N);
            } else {
                int64_t q = (j->kind == TCO_I8) ? ((const int8_t*)j->v)[i] : ((const int16_t*)j->v)[i];
                uint64_t mag[FR_N] = {(uint64_t)(q < 0 ? -q : q), 0, 0, 0};
                if (q < 0) mod_neg(&FR, x, mag); else memcpy(x, mag, sizeof x);
            }
            mod_mul(&FR, t, x, j->ell + FR_N * k);
            mod_add(&FR, acc, acc, t);
        }
        to_le(j->out + 32 * o, acc, FR_N);
    }
    return 0;
}

static void contract_last(const void* v, int kind, size_t outer, size_t d, const uint8_t* ell_bytes, uint8_t* out,
                          int nthreads) {
    uint64_t* ell = (uint64_t*)malloc(sizeof(uint64_t) * FR_N * d);
    for (size_t k = 0; k < d; ++k) from_le(ell + FR_N * k, ell_bytes + 32 * k, FR_N);
    if (nthreads < 1) nthreads = 1;
    if ((size_t)nthreads > outer) nthreads = outer ? (int)outer : 1;
    ctr_job_t* jobs = (ctr_job_t*)calloc(nthreads, sizeof *jobs);
    pthread_t* th = (pthread_t*)calloc(nthreads, sizeof *th);
    for (int t = 0; t < nthreads; ++t) {
        jobs[t].v = v; jobs[t].kind = kind; jobs[t].d = d; jobs[t].ell = ell; jobs[t].out = out;
        jobs[t].lo = outer * t / nthreads; jobs[t].hi = outer * (t + 1) / nthreads;
        pthread_create(&th[t], 0, ctr_worker, &jobs[t]);
    }
    for (int t = 0; t < nthreads; ++t) pthread_join(th[t], 0);
    free(jobs); free(th); free(ell);
}

/* f_T(tau) = sum_i e(T[i]) prod_j ell_j[i_j]; ell = concatenation of the m per-axis vectors
 * (32 bytes per entry, axis 0 first).  Nested sums, last axis first. */
int tco_f_at_tau(const void* T, int kind, int m, const uint32_t* shape, const uint8_t* ell, int nthreads,
                 uint8_t out[32]) {
    tco_init();
    if (m < 1 || m > 4) return -1;
    size_t n = 1, off[4], total = 0;
    for (int j = 0; j < m; ++j) { off[j] = total; total += shape[j]; n *= shape[j]; }
    const void* cur = T;
    int cur_kind = kind;
    uint8_t* owned = 0;
    for (int j = m - 1; j >= 0; --j) {
        size_t d = shape[j], outer = n / d;
        uint8_t* nxt = (uint8_t*)malloc(32 * (outer ? outer : 1));
        contract_last(cur, cur_kind, outer, d, ell + 32 * off[j], nxt, nthreads);
        free(owned);
        owned = nxt; cur = nxt; cur_kind = TCO_FR; n = outer;
    }
    memcpy(out, owned, 32);
    free(owned);
    return 0;
}
