// Memory-safety run of the library's CPU build (every kernel lane by lane, device buffers = malloc blocks)
// under AddressSanitizer: an access outside a buffer that the GPU would perform silently, or fault on, stops
// this program.  Results are checked only for consistency between entry points (the oracle comparisons live in
// the Python tests); what matters here is that every index the kernels form stays inside its allocation.
//
// Built and run by tests/test_host_asan.py:
//   g++ -O1 -g -std=c++17 -DTC_HOST_EMU -DTC_FB_C=8 -fsanitize=address,undefined asan_driver.cpp
#include "../../paper_2602_12630_amd/csrc/tc_lib.cpp"

#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <random>
#include <vector>

#define CHECK(call)                                                                             \
    do {                                                                                        \
        int rc_ = (call);                                                                       \
        if (rc_ != TC_OK) {                                                                     \
            std::fprintf(stderr, "%s:%d: %s -> %d (%s)\n", __FILE__, __LINE__, #call, rc_,      \
                         ctx ? tc_last_error(ctx) : "");                                        \
            return 1;                                                                           \
        }                                                                                       \
    } while (0)
#define REQUIRE(cond)                                                                           \
    do {                                                                                        \
        if (!(cond)) {                                                                          \
            std::fprintf(stderr, "%s:%d: %s does not hold\n", __FILE__, __LINE__, #cond);       \
            return 1;                                                                           \
        }                                                                                       \
    } while (0)

// exact-size heap copies, so that the sanitizer sees the true end of every "device" buffer
template <class T>
static T* exact(const std::vector<T>& v) {
    T* p = (T*)std::malloc(v.size() * sizeof(T) + (v.empty() ? 1 : 0));
    if (!v.empty()) std::memcpy(p, v.data(), v.size() * sizeof(T));
    return p;
}

int main() {
    tc_ctx* ctx = nullptr;
    CHECK(tc_ctx_create(&ctx, 0, nullptr));
    uint8_t tau[4 * 32] = {0};
    for (int j = 0; j < 4; ++j) {          // small trapdoors well off every grid used below
        tau[32 * j] = (uint8_t)(101 + j);
        tau[32 * j + 1] = 0x77;
        tau[32 * j + 5] = (uint8_t)(3 + j);
    }
    std::mt19937 rng(12345);
    tc_vk* vk = nullptr;
    CHECK(tc_vk_from_trapdoor(tau, 4, &vk));

    // --- flat commitments: ragged tiles, odd offsets, a batch with enough windows for the packed bucket sums
    {
        const uint32_t shape[2] = {37, 113};
        const size_t n = 37 * 113;
        tc_srs* srs = nullptr;
        CHECK(tc_setup_from_trapdoor(ctx, tau, 2, shape, TC_SRS_SUFFIX, &srs));
        std::vector<int16_t> x16(n);
        std::vector<int8_t> x8(n);
        for (size_t i = 0; i < n; ++i) {
            x16[i] = (int16_t)(rng() % 65536 - 32768);
            x8[i] = (int8_t)(rng() % 256 - 128);
        }
        x16[0] = -32768; x16[1] = 32767; x16[2] = 0;
        uint8_t c_a[96], c_b[96];
        int16_t* d16 = exact(x16);
        CHECK(tc_commit(ctx, srs, d16, TC_I16, c_a));
        {   // the same values at an odd offset of a larger block
            std::vector<int16_t> padded(n + 3);
            std::memcpy(padded.data() + 3, x16.data(), n * 2);
            int16_t* dp = exact(padded);
            CHECK(tc_commit(ctx, srs, dp + 3, TC_I16, c_b));
            REQUIRE(std::memcmp(c_a, c_b, 96) == 0);
            std::free(dp);
        }
        int8_t* d8 = exact(x8);
        CHECK(tc_commit(ctx, srs, d8, TC_I8, c_b));
        {
            const tc_srs* many_srs[9];
            const void* many_x[9];
            int many_t[9];
            for (int i = 0; i < 9; ++i) { many_srs[i] = srs; many_x[i] = d16; many_t[i] = TC_I16; }
            std::vector<uint8_t> out(9 * 96);
            CHECK(tc_commit_batch(ctx, 9, many_srs, many_x, many_t, out.data()));
            for (int i = 0; i < 9; ++i) REQUIRE(std::memcmp(out.data() + 96 * i, c_a, 96) == 0);
        }
        // openings (the row route needs a larger leading slice: see below) and verification
        const uint32_t kappa[2] = {36, 112};
        uint8_t y[32], pi[2 * 96];
        CHECK(tc_open(ctx, srs, d16, TC_I16, kappa, y, pi));
        CHECK(tc_verify(ctx, vk, 2, shape, c_a, kappa, y, pi));
        pi[5] ^= 1;
        REQUIRE(tc_verify(ctx, vk, 2, shape, c_a, kappa, y, pi) != TC_OK);
        std::free(d16);
        std::free(d8);
        tc_srs_destroy(srs);
    }
    // --- openings by rows (two-digit difference problems, job lists) and full-width scalars
    {
        const uint32_t shape[2] = {6, 2048};
        const size_t n = 6 * 2048;
        tc_srs* srs = nullptr;
        CHECK(tc_setup_from_trapdoor(ctx, tau, 2, shape, TC_SRS_SUFFIX, &srs));
        std::vector<int16_t> x(n);
        for (auto& v : x) v = (int16_t)(rng() % 65536 - 32768);
        int16_t* d = exact(x);
        uint8_t c[96], y[32], pi[2 * 96];
        CHECK(tc_commit(ctx, srs, d, TC_I16, c));
        const uint32_t kappa[2] = {2, 2047};
        CHECK(tc_open(ctx, srs, d, TC_I16, kappa, y, pi));
        CHECK(tc_verify(ctx, vk, 2, shape, c, kappa, y, pi));
        std::free(d);
        tc_srs_destroy(srs);
    }
    // --- interpolation in the three forms, Algorithm 1
    {
        const uint32_t shape[3] = {5, 7, 3};
        const size_t n = 5 * 7 * 3;
        std::vector<int16_t> x(n);
        for (auto& v : x) v = (int16_t)(rng() % 2001 - 1000);
        int16_t* d = exact(x);
        std::vector<uint8_t> zero(32 * n, 0);
        uint8_t* co[3];
        for (int f = 0; f < 3; ++f) {
            co[f] = exact(zero);
            CHECK(tc_interpolate_form(ctx, 3, shape, d, TC_I16, f, co[f]));
        }
        REQUIRE(std::memcmp(co[0], co[1], 32 * n) == 0 && std::memcmp(co[0], co[2], 32 * n) == 0);
        uint8_t* q = exact(zero);
        uint8_t* r = exact(zero);
        for (int axis = 0; axis < 3; ++axis) CHECK(tc_divide_by_linear(ctx, 3, shape, co[0], axis, shape[axis] - 1, q, r));
        for (int f = 0; f < 3; ++f) std::free(co[f]);
        std::free(q);
        std::free(r);
        std::free(d);
    }
    // --- trees: entries tree with ragged grid, batched openings, batch verification, an update
    {
        const uint32_t node[2] = {2, 2};
        tc_srs* node_srs = nullptr;
        CHECK(tc_setup_from_trapdoor(ctx, tau, 2, node, TC_SRS_SUFFIX | TC_SRS_FIXED_BASE, &node_srs));
        const uint32_t grid[2] = {7, 13};
        const size_t n = 7 * 13;
        std::vector<int16_t> x(n);
        for (auto& v : x) v = (int16_t)(rng() % 65536 - 32768);
        int16_t* d = exact(x);
        tc_tree_desc desc;
        std::memset(&desc, 0, sizeof desc);
        desc.m = 2;
        desc.grid[0] = grid[0]; desc.grid[1] = grid[1];
        desc.node_shape[0] = 2; desc.node_shape[1] = 2;
        desc.node_srs = node_srs;
        desc.leaf_kind = TC_LEAF_ENTRIES;
        desc.d_payload = d;
        desc.dtype = TC_I16;
        tc_tree* tree = nullptr;
        CHECK(tc_terkle_build(ctx, &desc, &tree));
        uint8_t root[96];
        CHECK(tc_terkle_root(tree, root));
        const int count = 5;
        const uint32_t leaves[count * 2] = {0, 0, 6, 12, 3, 7, 6, 0, 0, 12};
        std::vector<tc_path> paths(count);
        std::vector<uint8_t> roots(96 * count), values(32 * count, 0);
        for (int i = 0; i < count; ++i) {
            CHECK(tc_path_from_grid(2, grid, node, TC_LEAF_ENTRIES, leaves + 2 * i, 0, nullptr, nullptr, &paths[i]));
            std::memcpy(roots.data() + 96 * i, root, 96);
        }
        const size_t stride = 4096;
        std::vector<uint8_t> proofs(stride * count);
        std::vector<size_t> lens(count, stride);
        CHECK(tc_terkle_open_batch(ctx, tree, count, leaves, nullptr, proofs.data(), stride, lens.data()));
        for (int i = 0; i < count; ++i) {          // the opened value of the last step is the leaf value
            REQUIRE(lens[i] >= 32 + 96 * 2);
            std::memcpy(values.data() + 32 * i, proofs.data() + stride * i + lens[i] - 32, 32);
        }
        std::vector<int> verdict(count, -99);
        CHECK(tc_verify_paths_batch(ctx, vk, count, paths.data(), roots.data(), values.data(), proofs.data(), stride,
                                    lens.data(), verdict.data()));
        for (int i = 0; i < count; ++i) REQUIRE(verdict[i] == TC_OK);
        CHECK(tc_verify_path(ctx, vk, &paths[1], root, values.data() + 32, proofs.data() + stride, lens[1]));
        // an update must give the root of a fresh build over the changed payload
        d[3 * 13 + 7] = (int16_t)(d[3 * 13 + 7] + 5);
        CHECK(tc_terkle_update(ctx, tree, leaves + 4, nullptr, 5));
        uint8_t root_updated[96], root_rebuilt[96];
        CHECK(tc_terkle_root(tree, root_updated));
        tc_tree* again = nullptr;
        CHECK(tc_terkle_build(ctx, &desc, &again));
        CHECK(tc_terkle_root(again, root_rebuilt));
        REQUIRE(std::memcmp(root_updated, root_rebuilt, 96) == 0);
        tc_tree_destroy(again);
        tc_tree_destroy(tree);

        // --- tensors tree: three leaf tensors of two shapes under one (2,2) node
        const uint32_t s_a[2] = {4, 300}, s_b[1] = {513};
        tc_srs *srs_a = nullptr, *srs_b = nullptr;
        CHECK(tc_setup_from_trapdoor(ctx, tau, 2, s_a, TC_SRS_SUFFIX, &srs_a));
        CHECK(tc_setup_from_trapdoor(ctx, tau, 1, s_b, TC_SRS_SUFFIX, &srs_b));
        std::vector<int16_t> ta(1200), tb(513);
        std::vector<int8_t> tc8(1200);
        for (auto& v : ta) v = (int16_t)(rng() % 65536 - 32768);
        for (auto& v : tb) v = (int16_t)(rng() % 65536 - 32768);
        for (auto& v : tc8) v = (int8_t)(rng() % 256 - 128);
        int16_t *da = exact(ta), *db = exact(tb);
        int8_t* dc = exact(tc8);
        const tc_srs* leaf_srs[3] = {srs_a, srs_b, srs_a};
        const void* leaf_x[3] = {da, db, dc};
        const int leaf_t[3] = {TC_I16, TC_I16, TC_I8};
        tc_tree_desc td;
        std::memset(&td, 0, sizeof td);
        td.m = 2;
        td.grid[0] = 1; td.grid[1] = 3;
        td.node_shape[0] = 2; td.node_shape[1] = 2;
        td.node_srs = node_srs;
        td.leaf_kind = TC_LEAF_TENSORS;
        td.leaf_srs = leaf_srs;
        td.d_leaf_scalars = leaf_x;
        td.leaf_dtype = leaf_t;
        tc_tree* tt = nullptr;
        CHECK(tc_terkle_build(ctx, &td, &tt));
        const uint32_t leaf_idx[2] = {0, 2}, inner_idx[2] = {3, 299};
        size_t plen = stride;
        CHECK(tc_terkle_open(ctx, tt, leaf_idx, inner_idx, proofs.data(), &plen));
        tc_path tp;
        CHECK(tc_path_from_grid(2, td.grid, node, TC_LEAF_TENSORS, leaf_idx, 2, s_a, inner_idx, &tp));
        CHECK(tc_terkle_root(tt, root));
        CHECK(tc_verify_path(ctx, vk, &tp, root, proofs.data() + plen - 32, proofs.data(), plen));
        tc_tree_destroy(tt);
        std::free(da); std::free(db); std::free(dc);
        tc_srs_destroy(srs_a);
        tc_srs_destroy(srs_b);
        std::free(d);
        tc_srs_destroy(node_srs);
    }
    // --- the carry-free field form on extreme operands: UBSan stops the run on a signed overflow of a column sum or
    //     of a limb, i.e. on a violated bound; the 28-bit-limb products must agree with the 32-bit routine
    {
        std::vector<fp_t> edge;
        auto from_words = [](std::initializer_list<uint32_t> w) { fp_t x = fe_zero<FpParams>(); int i = 0; for (uint32_t v : w) x.l[i++] = v; return x; };
        fp_t pm1, pm2, ones, half;
        for (int i = 0; i < 12; ++i) { pm1.l[i] = FpParams::MOD[i]; pm2.l[i] = FpParams::MOD[i]; ones.l[i] = i < 11 ? 0xFFFFFFFFu : 0x19FFFFFFu; half.l[i] = FpParams::HALF[i]; }
        pm1.l[0] -= 1;
        pm2.l[0] -= 2;
        edge.push_back(fe_zero<FpParams>());
        edge.push_back(from_words({1}));
        edge.push_back(pm1);
        edge.push_back(pm2);
        edge.push_back(ones);                                   // every 28-bit limb at its maximum, top limb as large as p allows
        edge.push_back(half);
        edge.push_back(fe_one<FpParams>());
        edge.push_back(from_words({0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0x10000000u}));
        edge.push_back(from_words({0xFFFFFFFFu, 0, 0xFFFFFFFFu, 0, 0xFFFFFFFFu, 0, 0xFFFFFFFFu, 0, 0xFFFFFFFFu, 0, 0xFFFFFFFFu, 0}));
        std::vector<uint32_t> a, b;
        for (const fp_t& x : edge)
            for (const fp_t& y : edge) {
                a.insert(a.end(), x.l, x.l + 12);
                b.insert(b.end(), y.l, y.l + 12);
            }
        for (int i = 0; i < 64; ++i)
            for (int j = 0; j < 12; ++j) {
                a.push_back(j < 11 ? (uint32_t)rng() : (uint32_t)rng() % 0x1A000000u);
                b.push_back(j < 11 ? (uint32_t)rng() : (uint32_t)rng() % 0x1A000000u);
            }
        const size_t n = a.size() / 12;
        uint32_t *da = exact(a), *db = exact(b);
        std::vector<std::vector<uint32_t>> out(14, std::vector<uint32_t>(a.size()));
        for (int op : {0, 1, 6, 7, 9, 10, 11, 12, 13}) {
            uint32_t* d = exact(out[op]);
            CHECK(tc_ctx_field_op(ctx, op, da, db, n, d));
            CHECK(tc_ctx_sync(ctx));
            std::memcpy(out[op].data(), d, out[op].size() * 4);
            std::free(d);
        }
        REQUIRE(out[9] == out[0]);                              // a b both ways
        REQUIRE(out[10] == out[1]);                             // a^2 both ways
        // (a - b)(a + b) = a^2 - b^2 needs b^2: the same call with the operands exchanged
        std::vector<uint32_t> bsq(a.size()), diff(a.size());
        {
            uint32_t* d = exact(bsq);
            CHECK(tc_ctx_field_op(ctx, 1, db, da, n, d));
            CHECK(tc_ctx_sync(ctx));
            uint32_t *e = exact(diff), *asq = exact(out[1]);
            CHECK(tc_ctx_field_op(ctx, 7, asq, d, n, e));
            CHECK(tc_ctx_sync(ctx));
            std::memcpy(diff.data(), e, diff.size() * 4);
            std::free(d);
            std::free(e);
            std::free(asq);
        }
        REQUIRE(out[11] == diff);
        std::free(da);
        std::free(db);
    }
    tc_vk_destroy(vk);
    tc_ctx_destroy(ctx);
    std::puts("asan driver: ok");
    return 0;
}
