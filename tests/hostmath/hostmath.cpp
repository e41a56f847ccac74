// Host build of the library's field / curve headers, exported for CPU-side tests.
// The same inline functions run inside the HIP kernels; compiling them with g++ lets
// the CPU test-suite check them against the oracle without a GPU.
#include <cstring>

#define TC_HOST_EMU 1
#include <vector>

#include "../../paper_2602_12630_amd/csrc/kernels.h"
#include "../../paper_2602_12630_amd/csrc/pairing.h"

using namespace tc;

static fp_t fp_load(const uint8_t* b) { uint32_t w[12]; memcpy(w, b, 48); return fe_from_limbs<FpParams>(w); }
static void fp_store(uint8_t* b, const fp_t& a) { fp_t p = fe_to_plain(a); memcpy(b, p.l, 48); }
static fr_t fr_load(const uint8_t* b) { uint32_t w[8]; memcpy(w, b, 32); return fe_from_limbs<FrParams>(w); }
static void fr_store(uint8_t* b, const fr_t& a) { fr_t p = fe_to_plain(a); memcpy(b, p.l, 32); }
static g1_affine pt_load(const uint8_t* b) { uint32_t w[24]; memcpy(w, b, 96); return affine_from_canonical(w); }
static void pt_store(uint8_t* b, const g1_affine& p) { uint32_t w[24]; affine_to_canonical(p, w); memcpy(b, w, 96); }

extern "C" {
void hm_fp_mul(const uint8_t* a, const uint8_t* b, uint8_t* o) { fp_store(o, fp_mul(fp_load(a), fp_load(b))); }
void hm_fp_mul_limbs32(const uint8_t* a, const uint8_t* b, uint8_t* o) { fp_store(o, fe_mul<FpParams>(fp_load(a), fp_load(b))); }
void hm_fp_mul_f64(const uint8_t* a, const uint8_t* b, uint8_t* o) { fp_store(o, fp_mul_f64(fp_load(a), fp_load(b))); }
void hm_fp_sqr_f64(const uint8_t* a, const uint8_t*, uint8_t* o) { fp_store(o, fp_sqr_f64(fp_load(a))); }
void hm_fp_add(const uint8_t* a, const uint8_t* b, uint8_t* o) { fp_store(o, fp_add(fp_load(a), fp_load(b))); }
void hm_fp_sub(const uint8_t* a, const uint8_t* b, uint8_t* o) { fp_store(o, fp_sub(fp_load(a), fp_load(b))); }
void hm_fp_inv(const uint8_t* a, uint8_t* o) { fp_store(o, fe_inv_fermat<FpParams>(fp_load(a))); }
void hm_fp_inv_binary(const uint8_t* a, uint8_t* o) { fp_store(o, fe_inv<FpParams>(fp_load(a))); }
void hm_fr_inv_binary(const uint8_t* a, uint8_t* o) { fr_store(o, fe_inv<FrParams>(fr_load(a))); }
void hm_fp_inv_gcd(const uint8_t* a, uint8_t* o) { fp_store(o, fe_inv_gcd<FpParams>(fp_load(a))); }
void hm_fr_inv_gcd(const uint8_t* a, uint8_t* o) { fr_store(o, fe_inv_gcd<FrParams>(fr_load(a))); }
void hm_fr_mul(const uint8_t* a, const uint8_t* b, uint8_t* o) { fr_store(o, fr_mul(fr_load(a), fr_load(b))); }
void hm_fr_add(const uint8_t* a, const uint8_t* b, uint8_t* o) { fr_store(o, fr_add(fr_load(a), fr_load(b))); }
void hm_fr_sub(const uint8_t* a, const uint8_t* b, uint8_t* o) { fr_store(o, fr_sub(fr_load(a), fr_load(b))); }
void hm_fr_from_i32(int32_t v, uint8_t* o) { fr_store(o, fe_from_i32<FrParams>(v)); }
// a + b through the XYZZ laws: mode 0 = mixed add (a accumulated from affine), 1 = full add
// with both operands pushed away from Z = 1 first (a = (a + g) - g style is avoided: we use 2a - a)
void hm_g1_add(const uint8_t* a, const uint8_t* b, int mode, uint8_t* o) {
    g1_affine A = pt_load(a), B = pt_load(b);
    g1_xyzz r;
    if (mode == 0) {
        r = xyzz_madd(xyzz_from_affine(A), B);
    } else if (mode == 1) {
        r = xyzz_add(xyzz_from_affine(A), xyzz_from_affine(B));
    } else {
        // non-trivial ZZ on both sides: A = 2A + (-A), B = 2B + (-B)
        g1_xyzz A2 = xyzz_madd(xyzz_dbl_affine(A), affine_neg(A));
        g1_xyzz B2 = xyzz_madd(xyzz_dbl(xyzz_from_affine(B)), affine_neg(B));
        r = xyzz_add(A2, B2);
    }
    pt_store(o, xyzz_to_affine(r));
}
void hm_g1_mul(const uint8_t* k, const uint8_t* p, uint8_t* o) {
    uint32_t w[8]; memcpy(w, k, 32);
    pt_store(o, xyzz_to_affine(xyzz_mul_affine(w, 256, pt_load(p))));
}
// sum of n points through the four-wave cooperative reduction, phases run lane by lane
struct ArraySrc {
    const g1_xyzz* in;
    uint32_t n;
    g1_xyzz* out;
    uint32_t count(uint32_t) const { return n; }
    g1_xyzz load(uint32_t, uint32_t i) const { return in[i]; }
    void store(uint32_t, const g1_xyzz& r) const { *out = r; }
};
void hm_coop_reduce(const uint8_t* pts, uint32_t n, int spread, uint8_t* o) {
    std::vector<g1_xyzz> in(n ? n : 1);
    for (uint32_t i = 0; i < n; ++i) {
        g1_affine a = pt_load(pts + 96 * (size_t)i);
        // spread = 1: operands away from ZZ = 1, as sums of sums are (2a - a)
        in[i] = spread ? xyzz_madd(xyzz_dbl_affine(a), affine_neg(a)) : xyzz_from_affine(a);
    }
    g1_xyzz r;
    typedef CoopReduce<ArraySrc> K;
    K k{ArraySrc{in.data(), n, &r}};
    std::vector<uint8_t> lds(K::LDS_BYTES);
    for (int ph = 0; ph < K::PHASES; ++ph)
        for (uint32_t lane = 0; lane < (uint32_t)K::BLOCK; ++lane) k.phase(ph, lane, 0, lds.data());
    pt_store(o, xyzz_to_affine(r));
}
// the verifier's short final exponentiation against the plain one: must be its cube; also x^p, x^(p^2) by powers
int hm_final_exponentiation_forms(const uint8_t* p, uint32_t k) {
    using namespace tc::pairing;
    uint32_t kk[1] = {k};
    g2_affine q = g2_mul(kk, 32, g2_generator());
    fp12 f = miller(pt_load(p), q);
    fp12 e1 = final_exponentiation(f), e3 = final_exponentiation_cubed(f);
    bool cube = f12_eq(f12_mul(f12_sqr(e1), e1), e3);
    // Frobenius maps on an arbitrary element (the Miller value): compare with plain powers by p and p^2
    fp12 xp = f12_one(), base = f;
    for (int i = 0; i < 12 * 32; ++i) {                      // p, bit by bit from the limbs of the modulus
        if ((FpParams::MOD[i >> 5] >> (i & 31)) & 1u) xp = f12_mul(xp, base);
        base = f12_sqr(base);
    }
    bool frob1 = f12_eq(xp, f12_frob1(f));
    bool frob2 = f12_eq(f12_frob1(f12_frob1(f)), f12_frob2(f));
    bool inv = f12_eq(f12_mul(f, f12_inv(f)), f12_one());
    return (cube ? 1 : 0) | (frob1 ? 2 : 0) | (frob2 ? 4 : 0) | (inv ? 8 : 0);
}
void hm_g1_generator(uint8_t* o) { pt_store(o, affine_generator()); }
void hm_phi(const uint8_t* p, uint8_t* o) { fr_t v = phi_map(pt_load(p)); memcpy(o, v.l, 32); }
}
