/*
 * Host side of libtc.so: the C ABI declared in include/tc.h.
 *
 * Everything that touches tensor data runs in the kernels of kernels.h; this
 * file plans launches, owns device memory and moves the few result bytes.
 * Compiled by hipcc for gfx950 (product) or, with -DTC_HOST_EMU, by g++ as a
 * lane-by-lane emulation used only by CPU tests of this host logic.
 */
#include <algorithm>
#include <new>
#include <random>
#include <string>
#include <thread>
#include <memory>
#include <mutex>
#include <vector>

#include "../../include/tc.h"
#include "kernels.h"
#include "pairing.h"
#include "selector.h"

using namespace tc;

/* Scratch memory of the entry point that allocates nothing (tc_commit_static): one array per GPU, part of the
 * code object, held until the process ends.  In host code the array's name is only a stand-in: the address on a
 * device comes from hipGetSymbolAddress, once per device, and only that pointer is ever handed to a kernel. */
#if defined(TC_HOST_EMU)
alignas(256) static uint8_t tc_static_scratch[TC_STATIC_SCRATCH_BYTES];
#else
static __device__ __align__(256) uint8_t tc_static_scratch[TC_STATIC_SCRATCH_BYTES];
#endif
static const int MAX_DEVICES = 64;
static std::mutex g_scratch_lock;
static uint8_t* g_scratch_ptr[MAX_DEVICES];        /* per device: where its copy of the array lives */
/* address of the static scratch on `device`, which must be the current device */
static int static_scratch_address(int device, uint8_t** out) {
    *out = nullptr;
    if (device < 0 || device >= MAX_DEVICES) return 1;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[device]) {
#if defined(TC_HOST_EMU)
        g_scratch_ptr[device] = tc_static_scratch;
#else
        void* ptr = nullptr;
        int e = (int)hipGetSymbolAddress(&ptr, HIP_SYMBOL(tc_static_scratch));
        if (e) return e;
        if (!ptr) return 1;
        g_scratch_ptr[device] = (uint8_t*)ptr;
#endif
    }
    *out = g_scratch_ptr[device];
    return 0;
}

/* ======================================================================================= */
/* objects                                                                                 */
/* ======================================================================================= */
struct Arena {
    uint8_t* base = nullptr;
    size_t cap = 0, off = 0, demand = 0;
    std::vector<void*> extra;
    bool fixed = false;            /* a block that never grows: a request that does not fit fails instead of allocating */
};

/* The level arrays of the last destroyed tree, kept for the next build: allocating and freeing device memory
 * costs more than a small tree's levels and waits for every stream of the device.  Shared by a context and
 * its trees, so that either may go first. */
struct TreePool {
    void* block = nullptr;
    size_t cap = 0;
    bool closed = false;
};

/* Pinned host memory that small host arrays pass through on their way to the device (job lists, tables of
 * pointers, verification steps): a copy from pageable memory makes the host wait until the stream has reached it,
 * a copy from pinned memory does not.  Slots are handed out in order and reused only after the stream has been
 * waited for. */
struct Staging {
    uint8_t* base = nullptr;
    size_t cap = 0, off = 0;
};

struct tc_ctx {
    std::shared_ptr<TreePool> tree_pool = std::make_shared<TreePool>();
    int device = 0;
    rt::stream_t stream = nullptr;
    std::string err;
    Arena ws;
    Arena ws_static;                   /* the device's static scratch array, for the entry point that allocates nothing */
    Arena* wsp = &ws;                  /* the workspace that the current call draws from */
    bool static_mode = false;          /* set for the duration of such a call: no allocation, no wait for the stream */
    Staging staging;
    g1_affine* gtable = nullptr;       /* fixed-base table of the generator */
    bool profiling = false;
    std::vector<std::pair<rt::event_t, rt::event_t>> prof[TC_PROF_KINDS];
    uint64_t prof_units[TC_PROF_KINDS] = {0, 0, 0, 0};
    int64_t opt[TC_OPT_COUNT] = {0, 0, 0, 0};      /* tuning options, 0 = automatic */
};

struct tc_srs {
    int m = 0;
    uint32_t shape[4] = {1, 1, 1, 1};
    uint32_t flags = 0;
    uint64_t n[4] = {0, 0, 0, 0};
    g1_affine* pts[4] = {nullptr, nullptr, nullptr, nullptr};
    g1_affine* fb[4] = {nullptr, nullptr, nullptr, nullptr};
    g1_affine* open_tab = nullptr;      /* U[kappa, t] of the leading axis (TC_SRS_OPEN_TABLE), n[0] points */
    bool shifted = false;               /* pts[0] has 2 n[0] points, the second half holding 2^8 times the first (TC_SRS_OPEN_TABLE) */
    uint8_t* pad0 = nullptr;            /* pts[0] (both halves) once more at a stride of 128 bytes: what the accumulation gathers from */
    fr_t* axis_mem = nullptr;
    AxisTables ax[4];
};

struct TreeLevel {
    uint32_t grid[4] = {1, 1, 1, 1};
    uint64_t n = 0;
    g1_affine* C = nullptr;
    fr_plain* phi = nullptr;
};

struct tc_tree {
    int m = 0;
    uint32_t grid[4] = {1, 1, 1, 1};
    uint32_t node_shape[4] = {1, 1, 1, 1};
    uint32_t B = 1;
    const tc_srs* node_srs = nullptr;
    int leaf_kind = 0;
    const void* d_payload = nullptr;
    int dtype = 0;
    std::vector<const tc_srs*> leaf_srs;
    std::vector<const void*> leaf_scalars;
    std::vector<int> leaf_dtype;
    std::vector<TreeLevel> levels;
    /* per leaf tensor: its row commitments once an opening has computed them (device memory, owned by the tree);
     * filled in by openings, which take the tree as const */
    mutable std::vector<g1_affine*> row_cache;
    void* block = nullptr;          /* one device allocation holds C and phi of every level */
    size_t block_cap = 0;
    std::shared_ptr<TreePool> pool;
    uint8_t root[96];
};

struct tc_vk {
    int m = 0;
    uint8_t tau[4][32];
    /* tau_i - (kappa + 1), split for the curve endomorphism, for the positions of small node shapes:
     * the steps of a tree path ask for the same few scalars over and over */
    static const uint32_t SPLIT_CACHE = 64;
    uint32_t k1[4][SPLIT_CACHE][4];
    uint32_t k2[4][SPLIT_CACHE][4];
};

/* ======================================================================================= */
/* helpers                                                                                 */
/* ======================================================================================= */
static int fail(tc_ctx* ctx, int code, const char* msg) {
    if (ctx) ctx->err = msg;
    return code;
}
static int fail_hip(tc_ctx* ctx, int e, const char* where) {
    if (ctx) ctx->err = std::string(where) + ": " + rt::error_string(e);
    return TC_ERR_HIP;
}
#define RT(call)                                             \
    do {                                                     \
        int e_ = (call);                                     \
        if (e_) return fail_hip(ctx, e_, #call);             \
    } while (0)
#define TRY(call)                 \
    do {                          \
        int rc_ = (call);         \
        if (rc_ != TC_OK) return rc_; \
    } while (0)

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

/* wait for the context's stream; every staged host array has been consumed by then */
static int ctx_sync(tc_ctx* ctx) {
    RT(rt::stream_sync(ctx->stream));
    ctx->staging.off = 0;
    return TC_OK;
}
/* dst (device) <- src (host, any memory, free again on return), asynchronous on the context's stream */
static int h2d(tc_ctx* ctx, void* dst, const void* src, size_t bytes) {
    if (!bytes) return TC_OK;
    Staging& S = ctx->staging;
    size_t need = (bytes + 63) / 64 * 64;
    if (S.off + need > S.cap) {
        TRY(ctx_sync(ctx));
        if (need > S.cap) {
            if (S.base) rt::host_pinned_free(S.base);
            S.base = nullptr;
            S.cap = 0;
            size_t want = std::max<size_t>(2 * need, (size_t)1 << 20);
            void* p = nullptr;
            if (rt::host_pinned_malloc(&p, want) != 0) return fail(ctx, TC_ERR_NOMEM, "pinned host allocation failed");
            S.base = (uint8_t*)p;
            S.cap = want;
        }
    }
    memcpy(S.base + S.off, src, bytes);
    RT(rt::memcpy_h2d(dst, S.base + S.off, bytes, ctx->stream));
    S.off += need;
    return TC_OK;
}

/* The same for a few words when the call may not allocate (the staging buffer may have to grow) nor wait: the
 * words travel as kernel arguments, one launch per PokeWords::MAXW of them. */
static int upload_small(tc_ctx* ctx, void* dst, const void* src, size_t bytes) {
    if (!ctx->static_mode) return h2d(ctx, dst, src, bytes);
    if (bytes % 4) return fail(ctx, TC_ERR_STATE, "internal: upload not a whole number of words");
    size_t words = bytes / 4;
    for (size_t i = 0; i < words; i += PokeWords::MAXW) {
        PokeWords k;
        k.dst = (uint32_t*)dst + i;
        k.n = (uint32_t)std::min<size_t>(PokeWords::MAXW, words - i);
        memset(k.w, 0, sizeof k.w);
        memcpy(k.w, (const uint8_t*)src + 4 * i, 4 * (size_t)k.n);
        RT(rt::launch<64>(k.n, ctx->stream, k));
    }
    return TC_OK;
}

/* Workspace: a slab that grows to the largest demand seen; within one API call allocations
 * are bump-pointer, overflow goes to one-off blocks released at the next reset. */
static int ws_reset(tc_ctx* ctx) {
    Arena& A = ctx->ws;
    if (!A.extra.empty() || A.demand > A.cap) {
        TRY(ctx_sync(ctx));
        for (void* p : A.extra) rt::dev_free(p);
        A.extra.clear();
        if (A.demand > A.cap) {
            if (A.base) rt::dev_free(A.base);
            A.base = nullptr;
            A.cap = 0;
            void* p = nullptr;
            size_t want = align_up(A.demand + A.demand / 8, 1 << 20);
            if (rt::dev_malloc(&p, want) == 0) {
                A.base = (uint8_t*)p;
                A.cap = want;
            }
        }
    }
    A.off = 0;
    A.demand = 0;
    return TC_OK;
}
static void* ws_alloc(tc_ctx* ctx, size_t bytes) {
    Arena& A = *ctx->wsp;
    bytes = align_up(bytes ? bytes : 1, 256);
    A.demand += bytes;
    if (A.off + bytes <= A.cap) {
        void* p = A.base + A.off;
        A.off += bytes;
        return p;
    }
    if (A.fixed) return nullptr;
    void* p = nullptr;
    if (rt::dev_malloc(&p, bytes) != 0) return nullptr;
    A.extra.push_back(p);
    return p;
}
template <class T>
static T* ws_array(tc_ctx* ctx, uint64_t count) {
    return (T*)ws_alloc(ctx, (size_t)count * sizeof(T));
}
#define WS(ptr, T, count)                                                   \
    T* ptr = ws_array<T>(ctx, (count));                                     \
    if (!ptr) return fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed")

static bool valid_dtype_scalar(int dt) { return dt == TC_I8 || dt == TC_I16 || dt == TC_FR; }
static size_t dtype_size(int dt) { return dt == TC_I8 ? 1 : dt == TC_I16 ? 2 : dt == TC_FR ? 32 : dt == TC_F16 ? 2 : 0; }

static bool shape_ok(int m, const uint32_t* shape, uint64_t* total) {
    if (m < 1 || m > TC_MAX_ORDER || !shape) return false;
    uint64_t n = 1;
    for (int j = 0; j < m; ++j) {
        if (shape[j] == 0) return false;
        n *= shape[j];
        if (n > (1ull << 31) - 1) return false;       /* point indices carry a sign bit */
    }
    if (total) *total = n;
    return true;
}

/* ---- host-side Fr helpers (setup only) ------------------------------------------------- */
static bool fr_bytes_canonical(const uint8_t* b, uint32_t* w) {
    memcpy(w, b, 32);
    return limbs_gt<8>(FrParams::MOD, w);
}
static void fr_batch_inverse(std::vector<fr_t>& v) {       /* every entry non-zero */
    size_t n = v.size();
    if (!n) return;
    std::vector<fr_t> pre(n);
    fr_t run = fe_one<FrParams>();
    for (size_t i = 0; i < n; ++i) {
        pre[i] = run;
        run = fr_mul(run, v[i]);
    }
    fr_t inv = fe_inv_fermat<FrParams>(run);
    for (size_t i = n; i-- > 0;) {
        fr_t vi = v[i];
        v[i] = fr_mul(inv, pre[i]);
        inv = fr_mul(inv, vi);
    }
}

/* ---- cooperative launches: a workgroup runs the phases of a functor with a barrier after each ---------- */
#if defined(TC_HOST_EMU)
template <int BLOCK, class F>
static int launch_coop(uint32_t groups, rt::stream_t, const F& f) {
    std::vector<uint8_t> lds(F::LDS_BYTES);
    for (uint32_t g = 0; g < groups; ++g)
        for (int ph = 0; ph < F::PHASES; ++ph)
            for (uint32_t lane = 0; lane < (uint32_t)BLOCK; ++lane) f.phase(ph, lane, g, lds.data());
    return 0;
}
#else
template <class F, int BLOCK>
__global__ __launch_bounds__(BLOCK) void coop_kernel(const F f) {
    extern __shared__ __align__(16) uint8_t lds[];
    for (int ph = 0; ph < F::PHASES; ++ph) {
        f.phase(ph, threadIdx.x, blockIdx.x, lds);
        __syncthreads();
    }
}
template <int BLOCK, class F>
static int launch_coop(uint32_t groups, rt::stream_t st, const F& f) {
    if (!groups) return 0;
    /* once per kernel, whichever host thread comes first (contexts of several threads share the kernels) */
    static std::once_flag attr_once;
    static int attr_error = 0;
    std::call_once(attr_once, [] {
        attr_error = (int)hipFuncSetAttribute(reinterpret_cast<const void*>(&coop_kernel<F, BLOCK>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)F::LDS_BYTES);
    });
    if (attr_error) return attr_error;
    hipLaunchKernelGGL((coop_kernel<F, BLOCK>), dim3(groups), dim3(BLOCK), F::LDS_BYTES, st, f);
    return (int)hipGetLastError();
}
#endif

/* cooperative launch whose number of phases is known only at run time */
#if defined(TC_HOST_EMU)
template <int BLOCK, class F>
static int launch_coop_n(uint32_t groups, rt::stream_t, const F& f, int phases) {
    std::vector<uint8_t> lds(F::LDS_BYTES);
    for (uint32_t g = 0; g < groups; ++g)
        for (int ph = 0; ph < phases; ++ph)
            for (uint32_t lane = 0; lane < (uint32_t)BLOCK; ++lane) f.phase(ph, lane, g, lds.data());
    return 0;
}
#else
template <class F, int BLOCK>
__global__ __launch_bounds__(BLOCK) void coop_kernel_n(const F f, int phases) {
    extern __shared__ __align__(16) uint8_t lds[];
    for (int ph = 0; ph < phases; ++ph) {
        f.phase(ph, threadIdx.x, blockIdx.x, lds);
        __syncthreads();
    }
}
template <int BLOCK, class F>
static int launch_coop_n(uint32_t groups, rt::stream_t st, const F& f, int phases) {
    if (!groups || phases <= 0) return 0;
    hipLaunchKernelGGL((coop_kernel_n<F, BLOCK>), dim3(groups), dim3(BLOCK), F::LDS_BYTES, st, f, phases);
    return (int)hipGetLastError();
}
#endif

/* ======================================================================================= */
/* context                                                                                 */
/* ======================================================================================= */
static bool option_value_ok(int option, int64_t v) {
    if (v == 0) return true;
    switch (option) {
        case TC_OPT_ACC_SUBRUN: return v >= 1 && v <= 64;
        case TC_OPT_ACC_FANIN: return v >= 2 && v <= 64;
        case TC_OPT_FR_WINDOW: return v == 8 || v == 16;
        case TC_OPT_CHECK_LEVEL: return v == 1;
        default: return false;
    }
}
extern "C" int tc_ctx_set_option(tc_ctx* ctx, int option, int64_t value) {
    if (!ctx) return TC_ERR_ARG;
    if (option < 0 || option >= TC_OPT_COUNT || !option_value_ok(option, value)) return fail(ctx, TC_ERR_ARG, "unknown option or value out of range");
    ctx->opt[option] = value;
    return TC_OK;
}
extern "C" int tc_ctx_get_option(const tc_ctx* ctx, int option, int64_t* value) {
    if (!ctx || !value || option < 0 || option >= TC_OPT_COUNT) return TC_ERR_ARG;
    *value = ctx->opt[option];
    return TC_OK;
}
static void options_from_environment(tc_ctx* ctx) {
    static const char* const names[TC_OPT_COUNT] = {"TC_ACC_SUBRUN", "TC_ACC_FANIN", "TC_FR_WINDOW", "TC_CHECK_LEVEL"};
    for (int o = 0; o < TC_OPT_COUNT; ++o) {
        const char* text = getenv(names[o]);
        if (!text || !*text) continue;
        char* end = nullptr;
        long long v = strtoll(text, &end, 10);
        if (end && *end == 0 && option_value_ok(o, (int64_t)v)) ctx->opt[o] = (int64_t)v;
    }
}

extern "C" int tc_ctx_create(tc_ctx** out, int device, void* hip_stream) {
    try {
        if (!out) return TC_ERR_ARG;
        *out = nullptr;
        tc_ctx* ctx = new (std::nothrow) tc_ctx();
        if (!ctx) return TC_ERR_NOMEM;
        ctx->device = device;
        ctx->stream = (rt::stream_t)hip_stream;
        int e = rt::set_device(device);
        if (e) {
            delete ctx;
            return TC_ERR_HIP;
        }
        /* probe: a tiny allocation proves that a device is really there */
        void* p = nullptr;
        if (rt::dev_malloc(&p, 256) != 0) {
            delete ctx;
            return TC_ERR_HIP;
        }
        rt::dev_free(p);
        /* this device's static scratch, for tc_commit_static */
        uint8_t* scratch = nullptr;
        if (static_scratch_address(device, &scratch) != 0) {
            delete ctx;
            return TC_ERR_HIP;
        }
        ctx->ws_static.base = scratch;
        ctx->ws_static.cap = TC_STATIC_SCRATCH_BYTES;
        ctx->ws_static.fixed = true;
        options_from_environment(ctx);
        *out = ctx;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}
extern "C" void tc_ctx_destroy(tc_ctx* ctx) {
    if (!ctx) return;
    rt::set_device(ctx->device);
    rt::stream_sync(ctx->stream);
    for (void* p : ctx->ws.extra) rt::dev_free(p);
    if (ctx->ws.base) rt::dev_free(ctx->ws.base);
    if (ctx->gtable) rt::dev_free(ctx->gtable);
    if (ctx->staging.base) rt::host_pinned_free(ctx->staging.base);
    if (ctx->tree_pool->block) rt::dev_free(ctx->tree_pool->block);
    ctx->tree_pool->block = nullptr;
    ctx->tree_pool->cap = 0;
    ctx->tree_pool->closed = true;
    for (auto& v : ctx->prof)
        for (auto& pr : v) { rt::event_destroy(pr.first); rt::event_destroy(pr.second); }
    delete ctx;
}
/* measurement hooks */
static void prof_begin(tc_ctx* ctx, int kind, rt::event_t* a, rt::event_t* b) {
    *a = *b = nullptr;
    if (!ctx->profiling || ctx->static_mode) return;
    if (rt::event_create(a) || rt::event_create(b)) return;
    rt::event_record(*a, ctx->stream);
    (void)kind;
}
static void prof_end(tc_ctx* ctx, int kind, rt::event_t a, rt::event_t b) {
    if (!ctx->profiling || ctx->static_mode || !a || !b) return;
    rt::event_record(b, ctx->stream);
    ctx->prof[kind].push_back({a, b});
}
extern "C" int tc_ctx_profile(tc_ctx* ctx, int enable) {
    try {
        if (!ctx) return TC_ERR_ARG;
        ctx->profiling = enable != 0;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}
extern "C" int tc_ctx_profile_read(tc_ctx* ctx, int kind, double* total_ms, uint64_t* launches) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (kind < 0 || kind >= TC_PROF_KINDS || !total_ms || !launches) return fail(ctx, TC_ERR_ARG, "bad argument");
        RT(rt::set_device(ctx->device));
        TRY(ctx_sync(ctx));
        double tot = 0;
        for (auto& pr : ctx->prof[kind]) {
            float ms = 0;
            RT(rt::event_elapsed_ms(pr.first, pr.second, &ms));
            tot += ms;
            rt::event_destroy(pr.first);
            rt::event_destroy(pr.second);
        }
        *total_ms = tot;
        *launches = ctx->prof[kind].size();
        ctx->prof[kind].clear();
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}
extern "C" int tc_ctx_profile_units(tc_ctx* ctx, int kind, uint64_t* units) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (kind < 0 || kind >= TC_PROF_KINDS || !units) return fail(ctx, TC_ERR_ARG, "bad argument");
        *units = ctx->prof_units[kind];
        ctx->prof_units[kind] = 0;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}
/* ---- measurement: what the integer ALUs sustain ------------------------------------------------------------
 * Register-only loops at a chosen number of waves per SIMD.  A workgroup is four waves, one per SIMD of a compute
 * unit; it asks for so much LDS that exactly `waves_per_simd` workgroups fit a compute unit, and the launch has
 * that many workgroups per compute unit, so every one of them is resident from start to end. */
#if !defined(TC_HOST_EMU)
template <int KIND>
__global__ __launch_bounds__(256) void alu_rate_kernel(uint32_t iters, uint32_t* sink) {
#if defined(__HIP_DEVICE_COMPILE__)          /* the body uses device-only instructions; the host pass needs the symbol alone */
    uint32_t t = blockIdx.x * 256u + threadIdx.x;
    uint32_t out = 0;
    if (KIND == TC_ALU_MAD || KIND == TC_ALU_MAD_CARRY) {
        /* eight independent chains, as the columns of a product give the scheduler independent work */
        uint64_t acc[8];
        uint32_t hi[8];
        uint32_t a = t * 2654435761u | 1u, b = (t + 12345u) * 40503u | 1u;
#pragma unroll
        for (int i = 0; i < 8; ++i) { acc[i] = t + (uint32_t)i; hi[i] = 0; }
        for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint64_t carry;
                asm volatile("v_mad_u64_u32 %0, %1, %2, %3, %0" : "+v"(acc[i]), "=s"(carry) : "v"(a), "v"(b));
                if (KIND == TC_ALU_MAD_CARRY) carry_into(hi[i], carry);     /* the third word of a 96-bit column sum */
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) out ^= (uint32_t)acc[i] ^ (uint32_t)(acc[i] >> 32) ^ hi[i];
    } else if (KIND == TC_ALU_FP28_MUL || KIND == TC_ALU_FP28_SQR) {
        fp28 x = fp28_one(), y = fp28_one();
        x.l[0] ^= (int32_t)(t & 0xFFFFu);
        y.l[1] ^= (int32_t)((t * 7u) & 0xFFFFu);
        for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll 1
            for (int i = 0; i < 8; ++i) x = KIND == TC_ALU_FP28_MUL ? fp28_mul(x, y) : fp28_sqr(x);
        }
#pragma unroll
        for (int i = 0; i < 14; ++i) out ^= (uint32_t)x.l[i];
    } else {
        fp_t x = fe_one<FpParams>(), y = fe_one<FpParams>();
        x.l[0] ^= t;
        y.l[1] ^= t * 7u;
        for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll 1
            for (int i = 0; i < 8; ++i)
                x = KIND == TC_ALU_FP_MUL ? fp_mul(x, y) : KIND == TC_ALU_FP_SQR ? fp_sqr(x) : KIND == TC_ALU_FP_MUL_F64 ? fp_mul_lat(x, y) : fp_sqr_lat(x);
        }
#pragma unroll
        for (int i = 0; i < 12; ++i) out ^= x.l[i];
    }
    if (out == 0x9E3779B9u) sink[0] = t;        /* keeps the loops alive; practically never taken */
#endif
}
#endif

extern "C" int tc_ctx_alu_rate(tc_ctx* ctx, int kind, int waves_per_simd, double* out_per_s) {
    if (!ctx) return TC_ERR_ARG;
    if (!out_per_s || kind < 0 || kind > TC_ALU_FP28_SQR) return fail(ctx, TC_ERR_ARG, "bad argument");
    if (waves_per_simd < 1 || waves_per_simd > 8) return fail(ctx, TC_ERR_ARG, "waves_per_simd must be 1..8");
#if defined(TC_HOST_EMU)
    return fail(ctx, TC_ERR_HIP, "no GPU in the host emulation");
#else
    RT(rt::set_device(ctx->device));
    hipDeviceProp_t prop;
    RT((int)hipGetDeviceProperties(&prop, ctx->device));
    uint32_t cus = (uint32_t)prop.multiProcessorCount;
    size_t lds_per_cu = prop.maxSharedMemoryPerMultiProcessor ? prop.maxSharedMemoryPerMultiProcessor : 65536;
    /* a workgroup may not ask for more than sharedMemPerBlock; one that asks for more than half the compute
     * unit's LDS still has the compute unit to itself */
    size_t lds = std::min<size_t>(lds_per_cu / (size_t)waves_per_simd, prop.sharedMemPerBlock) / 1024 * 1024;
    if (lds * ((size_t)waves_per_simd + 1) <= lds_per_cu) return fail(ctx, TC_ERR_STATE, "cannot pin that many waves per SIMD on this device");
    TRY(ws_reset(ctx));
    WS(sink, uint32_t, 1);
    uint32_t groups = cus * (uint32_t)waves_per_simd;
    bool mads = kind == TC_ALU_MAD || kind == TC_ALU_MAD_CARRY;
    uint32_t iters = mads ? 16384u : 256u;
    rt::event_t e0 = nullptr, e1 = nullptr;
    if (rt::event_create(&e0) || rt::event_create(&e1)) return fail(ctx, TC_ERR_HIP, "event creation failed");
    int rc = TC_OK;
    for (int rep = 0; rep < 2 && rc == TC_OK; ++rep) {       /* the first run warms up, the second is timed */
        rt::event_record(e0, ctx->stream);
        void (*k)(uint32_t, uint32_t*) = kind == TC_ALU_MAD         ? alu_rate_kernel<TC_ALU_MAD>
                                         : kind == TC_ALU_MAD_CARRY ? alu_rate_kernel<TC_ALU_MAD_CARRY>
                                         : kind == TC_ALU_FP_MUL    ? alu_rate_kernel<TC_ALU_FP_MUL>
                                         : kind == TC_ALU_FP_SQR    ? alu_rate_kernel<TC_ALU_FP_SQR>
                                         : kind == TC_ALU_FP_MUL_F64 ? alu_rate_kernel<TC_ALU_FP_MUL_F64>
                                         : kind == TC_ALU_FP_SQR_F64 ? alu_rate_kernel<TC_ALU_FP_SQR_F64>
                                         : kind == TC_ALU_FP28_MUL   ? alu_rate_kernel<TC_ALU_FP28_MUL>
                                                                     : alu_rate_kernel<TC_ALU_FP28_SQR>;
        int e = (int)hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (!e) {
            hipLaunchKernelGGL(k, dim3(groups), dim3(256), lds, ctx->stream, iters, sink);
            e = (int)hipGetLastError();
        }
        rt::event_record(e1, ctx->stream);
        if (e) rc = fail_hip(ctx, e, "alu_rate_kernel");
        if (rc == TC_OK && (e = rt::stream_sync(ctx->stream)) != 0) rc = fail_hip(ctx, e, "alu_rate_kernel");
    }
    float ms = 0;
    if (rc == TC_OK && rt::event_elapsed_ms(e0, e1, &ms) != 0) rc = fail(ctx, TC_ERR_HIP, "event timing failed");
    rt::event_destroy(e0);
    rt::event_destroy(e1);
    if (rc != TC_OK) return rc;
    double ops = (double)groups * 256.0 * (double)iters * 8.0;
    *out_per_s = ops / ((double)ms * 1e-3);
    return TC_OK;
#endif
}

extern "C" int tc_ctx_field_op(tc_ctx* ctx, int op, const void* d_a, const void* d_b, size_t n, void* d_out) {
    if (!ctx) return TC_ERR_ARG;
    if (op < 0 || op >= FOP_COUNT || ((!d_a || !d_b || !d_out) && n)) return fail(ctx, TC_ERR_ARG, "bad argument");
    if (n > 0xFFFFFFFFull) return fail(ctx, TC_ERR_SHAPE, "too many elements");
    RT(rt::set_device(ctx->device));
    RT(rt::launch<64>(n, ctx->stream, FieldOp{op, (const uint32_t*)d_a, (const uint32_t*)d_b, (uint32_t*)d_out}));
    return TC_OK;
}

extern "C" const char* tc_last_error(const tc_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }
extern "C" int tc_ctx_sync(tc_ctx* ctx) {
    try {
        if (!ctx) return TC_ERR_ARG;
        TRY(ctx_sync(ctx));
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ======================================================================================= */
/* normalisation and fixed-base tables                                                     */
/* ======================================================================================= */
static int normalize(tc_ctx* ctx, const g1_xyzz* d_in, uint64_t n, g1_affine* d_out) {
    uint32_t G = n >= (1u << 18) ? 8 : n >= (1u << 14) ? 2 : 1;
    BatchNormalize k{d_in, n, G, d_out};
    RT(rt::launch<64>((n + G - 1) / G, ctx->stream, k));
    return TC_OK;
}
/* XYZZ points on the device -> canonical bytes on the host */
static int points_to_host(tc_ctx* ctx, const g1_xyzz* d_in, uint32_t n, uint8_t* out) {
    WS(aff, g1_affine, n);
    WS(can, uint32_t, 24ull * n);
    TRY(normalize(ctx, d_in, n, aff));
    RT(rt::launch<64>(n, ctx->stream, ToCanonical{aff, can}));
    RT(rt::memcpy_d2h(out, can, 96ull * n, ctx->stream));
    TRY(ctx_sync(ctx));
    return TC_OK;
}
static int affine_to_host(tc_ctx* ctx, const g1_affine* d_in, uint32_t n, uint8_t* out) {
    WS(can, uint32_t, 24ull * n);
    RT(rt::launch<64>(n, ctx->stream, ToCanonical{d_in, can}));
    RT(rt::memcpy_d2h(out, can, 96ull * n, ctx->stream));
    TRY(ctx_sync(ctx));
    return TC_OK;
}

/* table[(k, w, j)] = j 2^(16 w) B_k for `nbases` affine bases already on the device */
static int build_fixed_base_table(tc_ctx* ctx, const g1_affine* d_bases, uint32_t nbases, g1_affine** out) {
    *out = nullptr;
    uint64_t entries = (uint64_t)nbases * FB_W * FB_NB;
    void* tab = nullptr;
    if (rt::dev_malloc(&tab, entries * sizeof(g1_affine)) != 0) return fail(ctx, TC_ERR_NOMEM, "fixed-base table allocation failed");
    g1_affine* table = (g1_affine*)tab;
    uint32_t nbw = nbases * FB_W;
    void *wbx = nullptr, *wba = nullptr, *tmp = nullptr;
    const uint32_t slab_bw = 32;                      /* window bases per slab: 32 * 32768 points */
    int rc = TC_OK;
    do {
        if (rt::dev_malloc(&wbx, (size_t)nbw * sizeof(g1_xyzz)) || rt::dev_malloc(&wba, (size_t)nbw * sizeof(g1_affine)) ||
            rt::dev_malloc(&tmp, (size_t)slab_bw * FB_NB * sizeof(g1_xyzz))) {
            rc = fail(ctx, TC_ERR_NOMEM, "fixed-base scratch allocation failed");
            break;
        }
        int e = rt::launch<64>(nbases, ctx->stream, FbWindowBases{d_bases, (g1_xyzz*)wbx});
        if (e) { rc = fail_hip(ctx, e, "FbWindowBases"); break; }
        rc = normalize(ctx, (g1_xyzz*)wbx, nbw, (g1_affine*)wba);
        if (rc) break;
        for (uint32_t bw0 = 0; bw0 < nbw && rc == TC_OK; bw0 += slab_bw) {
            uint32_t cnt = std::min(slab_bw, nbw - bw0);
            e = rt::launch<64>((uint64_t)cnt * (FB_NB / FB_CHUNK), ctx->stream, FbChunkFill{(g1_affine*)wba, bw0, (g1_xyzz*)tmp});
            if (e) { rc = fail_hip(ctx, e, "FbChunkFill"); break; }
            rc = normalize(ctx, (g1_xyzz*)tmp, (uint64_t)cnt * FB_NB, table + (uint64_t)bw0 * FB_NB);
        }
        if (rc) break;
        e = rt::stream_sync(ctx->stream);
        if (e) rc = fail_hip(ctx, e, "fixed-base table sync");
    } while (0);
    rt::stream_sync(ctx->stream);
    if (wbx) rt::dev_free(wbx);
    if (wba) rt::dev_free(wba);
    if (tmp) rt::dev_free(tmp);
    if (rc) {
        rt::dev_free(table);
        return rc;
    }
    *out = table;
    return TC_OK;
}

static int ensure_gtable(tc_ctx* ctx) {
    if (ctx->gtable) return TC_OK;
    g1_affine g = affine_generator();
    void* d = nullptr;
    if (rt::dev_malloc(&d, sizeof g) != 0) return fail(ctx, TC_ERR_NOMEM, "generator upload failed");
    int e = rt::memcpy_h2d(d, &g, sizeof g, ctx->stream);
    if (!e) e = rt::stream_sync(ctx->stream);
    int rc = e ? fail_hip(ctx, e, "generator upload") : build_fixed_base_table(ctx, (g1_affine*)d, 1, &ctx->gtable);
    rt::dev_free(d);
    return rc;
}

/* ======================================================================================= */
/* Setup                                                                                   */
/* ======================================================================================= */
extern "C" void tc_srs_destroy(tc_srs* srs) {
    if (!srs) return;
    for (int a = 0; a < 4; ++a) {
        if (srs->pts[a]) rt::dev_free(srs->pts[a]);
        if (srs->fb[a]) rt::dev_free(srs->fb[a]);
    }
    if (srs->axis_mem) rt::dev_free(srs->axis_mem);
    if (srs->open_tab) rt::dev_free(srs->open_tab);
    if (srs->pad0) rt::dev_free(srs->pad0);
    delete srs;
}
extern "C" uint64_t tc_srs_size(const tc_srs* srs, int first_axis) {
    if (!srs || first_axis < 0 || first_axis >= srs->m || !srs->pts[first_axis]) return 0;
    return srs->n[first_axis];
}

static const uint32_t FB_MAX_BASES = 64;

/* What Open needs per axis, public constants of the grid {1..d}: 1 / j, the barycentric weights of App. C
 * beta_i = 1 / prod_(k != i) (zeta_i - zeta_k) = (-1)^(d-1-i) / (i! (d-1-i)!), and 1 / beta_i (Montgomery form). */
static void axis_constants(uint32_t d, std::vector<fr_t>& inv_int, std::vector<fr_t>& beta, std::vector<fr_t>& beta_inv) {
    std::vector<fr_t> fact(d);
    inv_int.resize(d);
    beta.resize(d);
    beta_inv.resize(d);
    fact[0] = fe_one<FrParams>();
    for (uint32_t i = 1; i < d; ++i) fact[i] = fr_mul(fact[i - 1], fe_from_u32<FrParams>(i));
    for (uint32_t i = 0; i < d; ++i) {
        fr_t den = fr_mul(fact[i], fact[d - 1 - i]);
        if ((d - 1 - i) & 1u) den = fr_neg(den);
        beta_inv[i] = den;
        beta[i] = den;
        inv_int[i] = fe_from_u32<FrParams>(i ? i : 1);
    }
    fr_batch_inverse(beta);
    fr_batch_inverse(inv_int);
}
/* puts those tables of every axis of srs->shape on the device (srs->axis_mem, srs->ax) */
static int srs_upload_axis_tables(tc_ctx* ctx, tc_srs* srs) {
    std::vector<fr_t> tab_all;
    size_t tab_off[4] = {0, 0, 0, 0};
    for (int j = 0; j < srs->m; ++j) {
        std::vector<fr_t> inv_int, beta, beta_inv;
        axis_constants(srs->shape[j], inv_int, beta, beta_inv);
        tab_off[j] = tab_all.size();
        tab_all.insert(tab_all.end(), inv_int.begin(), inv_int.end());
        tab_all.insert(tab_all.end(), beta.begin(), beta.end());
        tab_all.insert(tab_all.end(), beta_inv.begin(), beta_inv.end());
    }
    void* p = nullptr;
    if (rt::dev_malloc(&p, tab_all.size() * sizeof(fr_t)) != 0) return fail(ctx, TC_ERR_NOMEM, "SRS table allocation failed");
    srs->axis_mem = (fr_t*)p;
    int e = rt::memcpy_h2d(p, tab_all.data(), tab_all.size() * sizeof(fr_t), ctx->stream);
    if (!e) e = rt::stream_sync(ctx->stream);         /* tab_all goes out of scope on return */
    if (e) return fail_hip(ctx, e, "SRS table upload");
    for (int j = 0; j < srs->m; ++j) {
        uint32_t d = srs->shape[j];
        srs->ax[j].inv_int = srs->axis_mem + tab_off[j];
        srs->ax[j].beta = srs->axis_mem + tab_off[j] + d;
        srs->ax[j].beta_inv = srs->axis_mem + tab_off[j] + 2 * (size_t)d;
    }
    return TC_OK;
}
static bool srs_flags_ok(uint32_t flags) {
    if (flags & ~(TC_SRS_SUFFIX | TC_SRS_FIXED_BASE | TC_SRS_MONOMIAL | TC_SRS_OPEN_TABLE)) return false;
    return !(flags & TC_SRS_MONOMIAL) || flags == TC_SRS_MONOMIAL;
}

/* Fills the second half of srs->pts[0] (allocated with 2 n[0] points) with 2^8 times the first: the row commitments
 * of an int16 tensor then need one window of 128 buckets per row for both 8-bit digits of an entry (the high digit
 * of entry i is entered as point n[0] + i), which halves the buckets that are reduced per row.  A public image of the
 * SRS; not stored in the SRS file, the import computes it again.  `tmp` holds at least min(slab, n[0]) XYZZ points. */
static const int SHIFT_BITS = 8;
static int srs_build_shifted_half(tc_ctx* ctx, tc_srs* srs, g1_xyzz* tmp, uint64_t slab) {
    uint64_t n0 = srs->n[0];
    for (uint64_t i0 = 0; i0 < n0; i0 += slab) {
        uint64_t cnt = std::min(slab, n0 - i0);
        RT(rt::launch<64>(cnt, ctx->stream, ShiftPoints{srs->pts[0] + i0, SHIFT_BITS, tmp}));
        TRY(normalize(ctx, tmp, cnt, srs->pts[0] + n0 + i0));
    }
    srs->shifted = true;
    return TC_OK;
}

/* the copy of pts[0] (with its shifted half, if any) at a stride of 128 bytes; without memory for it the
 * accumulation gathers from pts[0] itself */
static int srs_build_padded_copy(tc_ctx* ctx, tc_srs* srs) {
    uint64_t count = srs->n[0] * (srs->shifted ? 2 : 1);
    if (count > 0xFFFFFFFFull) return TC_OK;
    void* q = nullptr;
    if (rt::dev_malloc(&q, (size_t)count * PADDED_STRIDE) != 0) return TC_OK;
    srs->pad0 = (uint8_t*)q;
    RT(rt::launch<256>(count, ctx->stream, PadPoints{srs->pts[0], srs->pad0}));
    return TC_OK;
}
/* the table that a launch gathers the points i0 .. of S^(0) from, tagged with its stride */
static const g1_affine* srs_gather_table(const tc_srs* srs, uint64_t i0) {
    if (srs->pad0) return tag_padded(srs->pad0 + i0 * PADDED_STRIDE);
    return srs->pts[0] + i0;
}

extern "C" int tc_setup_from_trapdoor(tc_ctx* ctx, const uint8_t* tau, int m, const uint32_t* shape, uint32_t flags,
                                      tc_srs** out) {
    try {
        if (!ctx || !tau || !out) return ctx ? fail(ctx, TC_ERR_ARG, "null argument") : TC_ERR_ARG;
        *out = nullptr;
        uint64_t total = 0;
        if (!shape_ok(m, shape, &total)) return fail(ctx, TC_ERR_SHAPE, "bad shape");
        if (!srs_flags_ok(flags)) return fail(ctx, TC_ERR_ARG, "unknown flag, or the monomial SRS combined with another flag");
        if ((flags & TC_SRS_FIXED_BASE) && total > FB_MAX_BASES)
            return fail(ctx, TC_ERR_SHAPE, "fixed-base tables are limited to shapes with at most 64 entries");
        if ((flags & TC_SRS_OPEN_TABLE) && (m < 2 || shape[0] < 2)) return fail(ctx, TC_ERR_SHAPE, "the opening table needs a shape of order >= 2");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));

        /* per-axis Lagrange values at tau_j (barycentric form, App. C) */
        std::vector<fr_t> ell_all;
        uint32_t ell_off[4] = {0, 0, 0, 0};
        for (int j = 0; j < m; ++j) {
            uint32_t w[8];
            if (!fr_bytes_canonical(tau + 32 * j, w)) return fail(ctx, TC_ERR_RANGE, "trapdoor is not a canonical Fr element");
            bool small = true;
            for (int i = 1; i < 8; ++i) small = small && w[i] == 0;
            if (small && w[0] <= shape[j]) return fail(ctx, TC_ERR_RANGE, "trapdoor is zero or lies on the grid");
            uint32_t d = shape[j];
            fr_t t = fe_from_limbs<FrParams>(w);
            std::vector<fr_t> inv_int, beta, beta_inv, diff_inv(d), term(d);
            axis_constants(d, inv_int, beta, beta_inv);
            for (uint32_t i = 0; i < d; ++i) diff_inv[i] = fr_sub(t, fe_from_u32<FrParams>(i + 1));
            fr_batch_inverse(diff_inv);
            fr_t sum = fe_zero<FrParams>();
            for (uint32_t i = 0; i < d; ++i) {
                term[i] = fr_mul(beta[i], diff_inv[i]);
                sum = fr_add(sum, term[i]);
            }
            fr_t sum_inv = fe_inv_fermat<FrParams>(sum);
            ell_off[j] = (uint32_t)ell_all.size();
            if (flags & TC_SRS_MONOMIAL) {
                /* the same generator kernel multiplies per-axis factors: powers of tau_j give the monomial SRS */
                fr_t pw = fe_one<FrParams>();
                for (uint32_t i = 0; i < d; ++i) {
                    ell_all.push_back(pw);
                    pw = fr_mul(pw, t);
                }
            } else {
                for (uint32_t i = 0; i < d; ++i) ell_all.push_back(fr_mul(term[i], sum_inv));
            }
        }

        TRY(ensure_gtable(ctx));
        tc_srs* srs = new (std::nothrow) tc_srs();
        if (!srs) return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
        srs->m = m;
        srs->flags = flags;
        for (int j = 0; j < m; ++j) srs->shape[j] = shape[j];
        int rc = TC_OK;
        void* d_ell = nullptr;
        do {
            rc = srs_upload_axis_tables(ctx, srs);
            if (rc) break;
            /* behind the Lagrange values: room for the factors g(kappa) of the opening table */
            if (rt::dev_malloc(&d_ell, (ell_all.size() + shape[0]) * sizeof(fr_t)) != 0) {
                rc = fail(ctx, TC_ERR_NOMEM, "SRS table allocation failed");
                break;
            }
            int e = rt::memcpy_h2d(d_ell, ell_all.data(), ell_all.size() * sizeof(fr_t), ctx->stream);
            if (!e) e = rt::stream_sync(ctx->stream);
            if (e) { rc = fail_hip(ctx, e, "SRS table upload"); break; }
            int last_axis = (flags & TC_SRS_SUFFIX) ? m - 1 : 0;
            const uint64_t slab = 1ull << 20;
            void* tmp = nullptr;
            if (rt::dev_malloc(&tmp, (size_t)std::min<uint64_t>(slab, total) * sizeof(g1_xyzz)) != 0) {
                rc = fail(ctx, TC_ERR_NOMEM, "SRS scratch allocation failed");
                break;
            }
            for (int a = 0; a <= last_axis && rc == TC_OK; ++a) {
                uint64_t na = 1;
                for (int j = a; j < m; ++j) na *= shape[j];
                srs->n[a] = na;
                void* q = nullptr;
                bool twice = a == 0 && (flags & TC_SRS_OPEN_TABLE) && na <= 0x3FFFFFFFull;      /* room for the shifted half */
                if (rt::dev_malloc(&q, (size_t)na * (twice ? 2 : 1) * sizeof(g1_affine)) != 0) { rc = fail(ctx, TC_ERR_NOMEM, "SRS allocation failed"); break; }
                srs->pts[a] = (g1_affine*)q;
                SrsGen gen;
                gen.shape.m = m;
                for (int j = 0; j < 4; ++j) { gen.shape.d[j] = j < m ? shape[j] : 1; gen.ell_off[j] = ell_off[j]; }
                gen.first_axis = a;
                gen.ell = (const fr_t*)d_ell;
                gen.gtable = ctx->gtable;
                gen.out = (g1_xyzz*)tmp;
                for (uint64_t i0 = 0; i0 < na && rc == TC_OK; i0 += slab) {
                    uint64_t cnt = std::min(slab, na - i0);
                    gen.i0 = i0;
                    e = rt::launch<64>(cnt, ctx->stream, gen);
                    if (e) { rc = fail_hip(ctx, e, "SrsGen"); break; }
                    rc = normalize(ctx, (g1_xyzz*)tmp, cnt, srs->pts[a] + i0);
                }
                if (rc == TC_OK && (flags & TC_SRS_FIXED_BASE)) rc = build_fixed_base_table(ctx, srs->pts[a], (uint32_t)na, &srs->fb[a]);
                if (rc == TC_OK && twice) rc = srs_build_shifted_half(ctx, srs, (g1_xyzz*)tmp, std::min<uint64_t>(slab, total));
                if (rc == TC_OK && a == 0 && !(flags & TC_SRS_MONOMIAL)) rc = srs_build_padded_copy(ctx, srs);
            }
            if (rc == TC_OK && (flags & TC_SRS_OPEN_TABLE)) {
                /* U = the generator run once more with g(kappa) in the place of the leading axis' Lagrange values */
                fr_t* g = (fr_t*)d_ell + ell_all.size();
                void* q = nullptr;
                e = rt::launch<64>(shape[0], ctx->stream, OpenTableFactors{(const fr_t*)d_ell + ell_off[0], srs->ax[0].inv_int, shape[0], g});
                if (e) rc = fail_hip(ctx, e, "OpenTableFactors");
                else if (rt::dev_malloc(&q, (size_t)total * sizeof(g1_affine)) != 0) rc = fail(ctx, TC_ERR_NOMEM, "opening table allocation failed");
                srs->open_tab = (g1_affine*)q;
                SrsGen gen;
                gen.shape.m = m;
                for (int j = 0; j < 4; ++j) { gen.shape.d[j] = j < m ? shape[j] : 1; gen.ell_off[j] = ell_off[j]; }
                gen.ell_off[0] = (uint32_t)ell_all.size();
                gen.first_axis = 0;
                gen.ell = (const fr_t*)d_ell;
                gen.gtable = ctx->gtable;
                gen.out = (g1_xyzz*)tmp;
                for (uint64_t i0 = 0; i0 < total && rc == TC_OK; i0 += slab) {
                    uint64_t cnt = std::min(slab, total - i0);
                    gen.i0 = i0;
                    e = rt::launch<64>(cnt, ctx->stream, gen);
                    if (e) { rc = fail_hip(ctx, e, "SrsGen"); break; }
                    rc = normalize(ctx, (g1_xyzz*)tmp, cnt, srs->open_tab + i0);
                }
            }
            e = rt::stream_sync(ctx->stream);
            if (e && rc == TC_OK) rc = fail_hip(ctx, e, "SRS generation");
            rt::dev_free(tmp);
        } while (0);
        if (d_ell) rt::dev_free(d_ell);
        if (rc != TC_OK) {
            tc_srs_destroy(srs);
            return rc;
        }
        *out = srs;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ---- the public parameters as a flat file (Def. 4.1, Setup publishes pp = (srs, Omega)) ----------------------
 * Header (little-endian), then the tables S^(0) .. S^(last) one after the other, canonical 96-byte points:
 *     0  char[8]  "TCSRS\0\0\0"
 *     8  u32      format version (1)
 *    12  u32      curve (1 = BLS12-381, points in G1)
 *    16  u32      basis (0 = Lagrange image of the monomial SRS on the grid prod {1..d_j}, 1 = monomial)
 *    20  u32      flags the SRS was built with (suffix tables are stored, fixed-base tables are rebuilt on import)
 *    24  u32      m
 *    28  u32[4]   shape (unused axes 1)
 *    44  u32      reserved (0)
 *    48  u64      number of points that follow
 *    56  ...      points */
static const char SRS_MAGIC[8] = {'T', 'C', 'S', 'R', 'S', 0, 0, 0};
static const size_t SRS_HEADER_BYTES = 56;
static const uint32_t FILE_VERSION = 1, CURVE_BLS12_381_G1 = 1;
/* points move between the device and the caller's buffer in pieces of this many */
static const uint64_t IO_CHUNK_POINTS = 1ull << 18;

static void put_u32(uint8_t* p, uint32_t v) { memcpy(p, &v, 4); }
static void put_u64(uint8_t* p, uint64_t v) { memcpy(p, &v, 8); }
static uint32_t get_u32(const uint8_t* p) { uint32_t v; memcpy(&v, p, 4); return v; }
static uint64_t get_u64(const uint8_t* p) { uint64_t v; memcpy(&v, p, 8); return v; }

/* device affine points -> canonical bytes in host memory, in pieces through the workspace */
static int export_points(tc_ctx* ctx, const g1_affine* d_pts, uint64_t n, uint8_t* out) {
    uint64_t chunk = std::min<uint64_t>(n ? n : 1, IO_CHUNK_POINTS);
    WS(can, uint32_t, 24ull * chunk);
    for (uint64_t i0 = 0; i0 < n; i0 += chunk) {
        uint64_t cnt = std::min(chunk, n - i0);
        RT(rt::launch<64>(cnt, ctx->stream, ToCanonical{d_pts + i0, can}));
        RT(rt::memcpy_d2h(out + 96ull * i0, can, 96ull * cnt, ctx->stream));
        TRY(ctx_sync(ctx));                      /* the piece of workspace is reused */
    }
    return TC_OK;
}
/* canonical bytes in host memory -> device affine points; every point must be canonical and on the curve */
static int import_points(tc_ctx* ctx, const uint8_t* in, uint64_t n, g1_affine* d_pts) {
    uint64_t chunk = std::min<uint64_t>(n ? n : 1, IO_CHUNK_POINTS);
    WS(can, uint32_t, 24ull * chunk);
    WS(d_ok, uint32_t, 1);
    RT(rt::launch<64>(1, ctx->stream, Fill32{d_ok, 1u}));
    for (uint64_t i0 = 0; i0 < n; i0 += chunk) {
        uint64_t cnt = std::min(chunk, n - i0);
        RT(rt::memcpy_h2d(can, in + 96ull * i0, 96ull * cnt, ctx->stream));
        RT(rt::launch<64>(cnt, ctx->stream, FromCanonicalChecked{can, d_pts + i0, d_ok}));
        TRY(ctx_sync(ctx));                      /* the caller's buffer may be pageable: the copy has read it by now */
    }
    uint32_t ok = 0;
    RT(rt::memcpy_d2h(&ok, d_ok, 4, ctx->stream));
    TRY(ctx_sync(ctx));
    if (!ok) return fail(ctx, TC_ERR_RANGE, "a point is not canonical or not on the curve");
    return TC_OK;
}

extern "C" int tc_srs_export(tc_ctx* ctx, const tc_srs* srs, void* host_buf, size_t* len) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!srs || !len) return fail(ctx, TC_ERR_ARG, "null argument");
        uint64_t count = 0;
        for (int a = 0; a < srs->m; ++a)
            if (srs->pts[a]) count += srs->n[a];
        if (srs->open_tab) count += srs->n[0];
        size_t need = SRS_HEADER_BYTES + 96 * (size_t)count;
        size_t cap = *len;
        *len = need;
        if (!host_buf) return TC_OK;                /* size query */
        if (cap < need) return fail(ctx, TC_ERR_ARG, "buffer too small for the SRS (needed size returned in *len)");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        uint8_t* o = (uint8_t*)host_buf;
        memset(o, 0, SRS_HEADER_BYTES);
        memcpy(o, SRS_MAGIC, 8);
        put_u32(o + 8, FILE_VERSION);
        put_u32(o + 12, CURVE_BLS12_381_G1);
        put_u32(o + 16, (srs->flags & TC_SRS_MONOMIAL) ? 1u : 0u);
        put_u32(o + 20, srs->flags);
        put_u32(o + 24, (uint32_t)srs->m);
        for (int j = 0; j < 4; ++j) put_u32(o + 28 + 4 * j, j < srs->m ? srs->shape[j] : 1u);
        put_u64(o + 48, count);
        o += SRS_HEADER_BYTES;
        for (int a = 0; a < srs->m; ++a) {
            if (!srs->pts[a]) continue;
            TRY(export_points(ctx, srs->pts[a], srs->n[a], o));
            o += 96 * (size_t)srs->n[a];
        }
        if (srs->open_tab) TRY(export_points(ctx, srs->open_tab, srs->n[0], o));
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

extern "C" int tc_srs_import(tc_ctx* ctx, const void* host_buf, size_t len, tc_srs** out) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!host_buf || !out) return fail(ctx, TC_ERR_ARG, "null argument");
        *out = nullptr;
        const uint8_t* in = (const uint8_t*)host_buf;
        if (len < SRS_HEADER_BYTES) return fail(ctx, TC_ERR_ARG, "SRS file truncated: no complete header");
        if (memcmp(in, SRS_MAGIC, 8) != 0) return fail(ctx, TC_ERR_ARG, "not an SRS file");
        if (get_u32(in + 8) != FILE_VERSION) return fail(ctx, TC_ERR_ARG, "unknown SRS file version");
        if (get_u32(in + 12) != CURVE_BLS12_381_G1) return fail(ctx, TC_ERR_ARG, "the SRS file is for another curve");
        uint32_t basis = get_u32(in + 16), flags = get_u32(in + 20), m = get_u32(in + 24);
        uint32_t shape[4];
        for (int j = 0; j < 4; ++j) shape[j] = get_u32(in + 28 + 4 * j);
        uint64_t count = get_u64(in + 48), total = 0;
        if (m < 1 || m > TC_MAX_ORDER || !shape_ok((int)m, shape, &total)) return fail(ctx, TC_ERR_SHAPE, "bad shape in the SRS file");
        for (uint32_t j = m; j < 4; ++j)
            if (shape[j] != 1) return fail(ctx, TC_ERR_SHAPE, "bad shape in the SRS file");
        if (!srs_flags_ok(flags) || basis > 1 || (basis == 1) != ((flags & TC_SRS_MONOMIAL) != 0))
            return fail(ctx, TC_ERR_ARG, "bad flags or basis kind in the SRS file");
        if ((flags & TC_SRS_FIXED_BASE) && total > FB_MAX_BASES)
            return fail(ctx, TC_ERR_SHAPE, "fixed-base tables are limited to shapes with at most 64 entries");
        if ((flags & TC_SRS_OPEN_TABLE) && (m < 2 || shape[0] < 2)) return fail(ctx, TC_ERR_SHAPE, "the opening table needs a shape of order >= 2");
        int last_axis = (flags & TC_SRS_SUFFIX) ? (int)m - 1 : 0;
        uint64_t expect = 0, n[4] = {0, 0, 0, 0};
        for (int a = 0; a <= last_axis; ++a) {
            n[a] = 1;
            for (uint32_t j = (uint32_t)a; j < m; ++j) n[a] *= shape[j];
            expect += n[a];
        }
        if (flags & TC_SRS_OPEN_TABLE) expect += total;
        if (count != expect) return fail(ctx, TC_ERR_ARG, "point count in the SRS file does not match its shape and flags");
        if (len != SRS_HEADER_BYTES + 96 * (size_t)count) return fail(ctx, TC_ERR_ARG, "SRS file truncated or too long for its point count");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        tc_srs* srs = new (std::nothrow) tc_srs();
        if (!srs) return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
        srs->m = (int)m;
        srs->flags = flags;
        for (uint32_t j = 0; j < m; ++j) srs->shape[j] = shape[j];
        int rc = srs_upload_axis_tables(ctx, srs);
        const uint8_t* src = in + SRS_HEADER_BYTES;
        for (int a = 0; a <= last_axis && rc == TC_OK; ++a) {
            srs->n[a] = n[a];
            void* q = nullptr;
            bool twice = a == 0 && (flags & TC_SRS_OPEN_TABLE) && n[a] <= 0x3FFFFFFFull;
            if (rt::dev_malloc(&q, (size_t)n[a] * (twice ? 2 : 1) * sizeof(g1_affine)) != 0) { rc = fail(ctx, TC_ERR_NOMEM, "SRS allocation failed"); break; }
            srs->pts[a] = (g1_affine*)q;
            rc = import_points(ctx, src, n[a], srs->pts[a]);
            src += 96 * (size_t)n[a];
            if (rc == TC_OK && (flags & TC_SRS_FIXED_BASE)) rc = build_fixed_base_table(ctx, srs->pts[a], (uint32_t)n[a], &srs->fb[a]);
            if (rc == TC_OK && twice) {
                const uint64_t slab = std::min<uint64_t>(1ull << 20, n[a]);
                void* tmp = nullptr;
                if (rt::dev_malloc(&tmp, (size_t)slab * sizeof(g1_xyzz)) != 0) { rc = fail(ctx, TC_ERR_NOMEM, "SRS scratch allocation failed"); break; }
                rc = srs_build_shifted_half(ctx, srs, (g1_xyzz*)tmp, slab);
                int e = rt::stream_sync(ctx->stream);
                if (e && rc == TC_OK) rc = fail_hip(ctx, e, "shifted SRS half");
                rt::dev_free(tmp);
            }
            if (rc == TC_OK && a == 0 && !(flags & TC_SRS_MONOMIAL)) rc = srs_build_padded_copy(ctx, srs);
        }
        if (rc == TC_OK && (flags & TC_SRS_OPEN_TABLE)) {
            void* q = nullptr;
            if (rt::dev_malloc(&q, (size_t)total * sizeof(g1_affine)) != 0) rc = fail(ctx, TC_ERR_NOMEM, "opening table allocation failed");
            srs->open_tab = (g1_affine*)q;
            if (rc == TC_OK) rc = import_points(ctx, src, total, srs->open_tab);
        }
        if (rc == TC_OK && rt::stream_sync(ctx->stream) != 0) rc = fail(ctx, TC_ERR_HIP, "SRS import");      /* other contexts may use it next */
        if (rc != TC_OK) {
            rt::stream_sync(ctx->stream);
            tc_srs_destroy(srs);
            return rc;
        }
        *out = srs;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

extern "C" int tc_srs_get_point(tc_ctx* ctx, const tc_srs* srs, int first_axis, uint64_t index, uint8_t out_g1[96]) {
    try {
        if (!ctx || !srs || !out_g1) return ctx ? fail(ctx, TC_ERR_ARG, "null argument") : TC_ERR_ARG;
        if (first_axis < 0 || first_axis >= srs->m || !srs->pts[first_axis]) return fail(ctx, TC_ERR_STATE, "table not present");
        if (index >= srs->n[first_axis]) return fail(ctx, TC_ERR_RANGE, "index outside the table");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        return affine_to_host(ctx, srs->pts[first_axis] + index, 1, out_g1);
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ======================================================================================= */
/* encode                                                                                  */
/* ======================================================================================= */
static int encode_tensor(tc_ctx* ctx, const void* d_src, int src_dtype, size_t n, float inv_scale, const float* d_inv_scale,
                         void* d_dst) {
    if ((!d_src || !d_dst) && n) return fail(ctx, TC_ERR_ARG, "null buffer");
    if (n > 0xFFFFFFFFull) return fail(ctx, TC_ERR_SHAPE, "tensor too large");
    RT(rt::set_device(ctx->device));
    /* the bulk goes 16 bytes per lane when both buffers allow it, the remainder element by element */
    bool aligned = (((uintptr_t)d_src | (uintptr_t)d_dst) & 15u) == 0;
    switch (src_dtype) {
        case TC_F16: {
            if (!d_inv_scale && (!(inv_scale == inv_scale) || inv_scale < 0)) return fail(ctx, TC_ERR_RANGE, "inv_scale must be a non-negative number");
            size_t bulk = aligned ? n / 8 : 0;
            RT(rt::launch<256>(bulk, ctx->stream, EncodeF16x8{(const Words16*)d_src, (Words16*)d_dst, inv_scale, d_inv_scale}));
            RT(rt::launch<256>(n - 8 * bulk, ctx->stream,
                               EncodeF16{(const uint16_t*)d_src + 8 * bulk, (int16_t*)d_dst + 8 * bulk, inv_scale, d_inv_scale}));
            return TC_OK;
        }
        case TC_I8: {
            size_t bulk = aligned ? n / 16 : 0;
            RT(rt::launch<256>(bulk, ctx->stream, Copy128{(const Words16*)d_src, (Words16*)d_dst}));
            RT(rt::launch<256>(n - 16 * bulk, ctx->stream, Copy8{(const uint8_t*)d_src + 16 * bulk, (uint8_t*)d_dst + 16 * bulk}));
            return TC_OK;
        }
        case TC_I16: {
            size_t bulk = aligned ? n / 8 : 0;
            RT(rt::launch<256>(bulk, ctx->stream, Copy128{(const Words16*)d_src, (Words16*)d_dst}));
            RT(rt::launch<256>(n - 8 * bulk, ctx->stream, Copy16{(const uint16_t*)d_src + 8 * bulk, (uint16_t*)d_dst + 8 * bulk}));
            return TC_OK;
        }
        default:
            return fail(ctx, TC_ERR_ARG, "unsupported source dtype");
    }
}
extern "C" int tc_encode_tensor(tc_ctx* ctx, const void* d_src, int src_dtype, size_t n, float inv_scale, void* d_dst) {
    if (!ctx) return TC_ERR_ARG;
    return encode_tensor(ctx, d_src, src_dtype, n, inv_scale, nullptr, d_dst);
}
extern "C" int tc_encode_tensor_scaled(tc_ctx* ctx, const void* d_src, int src_dtype, size_t n, const float* d_inv_scale,
                                       void* d_dst) {
    if (!ctx) return TC_ERR_ARG;
    if (!d_inv_scale) return fail(ctx, TC_ERR_ARG, "null scale");
    return encode_tensor(ctx, d_src, src_dtype, n, 0.0f, d_inv_scale, d_dst);
}
/* at most this many workgroups take part in the maximum (each ends in one atomic): one per compute unit */
static const uint32_t ABSMAX_MAX_GROUPS = 256;
extern "C" int tc_quant_scale(tc_ctx* ctx, const void* d_src, size_t n, float* d_inv_scale) {
    if (!ctx) return TC_ERR_ARG;
    if (!d_inv_scale || (!d_src && n)) return fail(ctx, TC_ERR_ARG, "null buffer");
    if (((uintptr_t)d_src & 1u) || ((uintptr_t)d_inv_scale & 3u)) return fail(ctx, TC_ERR_ARG, "misaligned buffer");
    if (n > 0xFFFFFFFFull) return fail(ctx, TC_ERR_SHAPE, "tensor too large");
    RT(rt::set_device(ctx->device));
    uint32_t* result = (uint32_t*)d_inv_scale;
    RT(rt::launch<64>(1, ctx->stream, Fill32{result, 0u}));
    uint32_t groups = (uint32_t)std::min<uint64_t>(ABSMAX_MAX_GROUPS, (n / 8 + AbsMaxF16::BLOCK - 1) / AbsMaxF16::BLOCK);
    if (groups == 0) groups = 1;
    if (n) RT((launch_coop<AbsMaxF16::BLOCK>(groups, ctx->stream, AbsMaxF16{(const uint16_t*)d_src, (uint64_t)n, groups, result})));
    RT(rt::launch<64>(1, ctx->stream, InvScaleFromAbsMax{result}));
    return TC_OK;
}

/* ======================================================================================= */
/* MSM engine                                                                              */
/* ======================================================================================= */
/* a tree level of at most this many nodes (two workgroups per compute unit) takes the cooperative sums */
static const uint64_t COOP_LEVEL_NODES = 512;
/* a tree level spreads the windows of a child over lanes as long as it stays within this many lanes (two waves per SIMD) */
static const uint64_t SPLIT_LEVEL_LANES = 131072;

/* prefix sums of cnt (n entries): start, lstart (of ceil(cnt / L)); optional zeroing of a cursor array */
static int scan_counts(tc_ctx* ctx, const uint32_t* cnt, uint32_t n, uint32_t L, uint32_t* start, uint32_t* lstart,
                       uint32_t* zero_me, uint32_t* tot_a, uint32_t* tot_b, uint32_t* tot_max) {
    uint32_t nchunks = (n + SCAN_CHUNK - 1) / SCAN_CHUNK;
    if (n <= ScanSmall::MAX_N) {          /* few buckets: one workgroup, one launch; the totals land where the chunked scan leaves them */
        RT((launch_coop<ScanSmall::BLOCK>(1, ctx->stream,
                                          ScanSmall{cnt, n, L, start, lstart, zero_me, tot_a + nchunks, tot_b + nchunks, tot_max + nchunks})));
        return TC_OK;
    }
    RT(rt::launch<64>(nchunks, ctx->stream, ScanChunkTotals{cnt, n, L, tot_a, tot_b, tot_max}));
    RT((launch_coop<ScanChunkOffsets::BLOCK>(1, ctx->stream, ScanChunkOffsets{nchunks, tot_a, tot_b, tot_max})));
    RT(rt::launch<64>(nchunks, ctx->stream, ScanWrite{cnt, n, L, tot_a, tot_b, nchunks, start, lstart, zero_me}));
    return TC_OK;
}

/* lanes of the bucket accumulation that are resident at once: 256 compute units x 4 SIMDs x 3 waves x 64 */
static const uint64_t ACC_RESIDENT_LANES = 256ull * 4 * 3 * 64;
/* from this many 128- or 256-bucket windows on (the row problems of openings), throughput matters and not depth */
#if defined(TC_HOST_EMU)
static const int SMALL_WINDOW_REDUCE_MIN = 8;          /* the CPU build of the tests reaches it with a handful of rows */
#else
static const int SMALL_WINDOW_REDUCE_MIN = 512;
#endif
/* from this many 32768-bucket windows on, a launch fills the chip with the packed row / column sums */
static const int ROWCOL_PACKED_WINDOWS = 8;

/* sum_k k B_k for every window of `bucket` (W windows of nb buckets) -> wsum[W] */
static int reduce_windows(tc_ctx* ctx, const g1_xyzz* bucket, int W, uint32_t nb, g1_xyzz* wsum) {
    if ((nb == 256 || nb == 128) && W >= SMALL_WINDOW_REDUCE_MIN) {
        /* many small windows (row problems of openings): throughput matters, not depth */
        StridedSums S{bucket, nb, (uint32_t)W, nullptr, nullptr, nullptr};
        uint64_t lanes = S.lanes();
        if (lanes > 0xFFFFFFF0ull) return fail(ctx, TC_ERR_SHAPE, "too many windows in one launch");
        WS(sums, g1_xyzz, lanes);
        WS(parts, g1_xyzz, 2ull * (uint32_t)W);
        WS(redo, uint32_t, lanes + 1);
        S.out = sums; S.redo_count = redo; S.redo_list = redo + 1;
        RT(rt::launch<64>(1, ctx->stream, Fill32{redo, 0u}));
        RT((rt::launch_waves<64, 2>(lanes, ctx->stream, S)));
        uint32_t redo_lanes = (uint32_t)std::min<uint64_t>(lanes, ACC_RESIDENT_LANES);
        RT(rt::launch<64>(redo_lanes, ctx->stream, StridedRedo<StridedSums>{S, redo_lanes}));
        RT(rt::launch<64>(2ull * (uint32_t)W, ctx->stream, SmallWeighted{sums, S.cols(), (uint32_t)W, parts}));
        RT(rt::launch<64>((uint32_t)W, ctx->stream, SmallFinish{parts, S.cols(), (uint32_t)W, wsum}));
        return TC_OK;
    }
    if (nb == 128 || nb == 256) {
        WS(w1, g1_xyzz, (uint32_t)W);
        WS(s1, g1_xyzz, (uint32_t)W);
        if (nb == 128) RT((launch_coop<128>((uint32_t)W, ctx->stream, WeightedBlockSum<128>{bucket, (uint32_t)W * nb, w1, s1, nullptr, 0})));
        else RT((launch_coop<256>((uint32_t)W, ctx->stream, WeightedBlockSum<256>{bucket, (uint32_t)W * nb, w1, s1, nullptr, 0})));
        RT(rt::launch<64>((uint32_t)W, ctx->stream, WindowFinish{w1, nullptr, nullptr, 1, 0, wsum}));
        return TC_OK;
    }
    if (nb != 32768) return fail(ctx, TC_ERR_STATE, "unsupported bucket count");
    /* 128 x 256 bucket matrix: row / column sums, then two small weighted sums per window */
    WS(rows, g1_xyzz, 512ull * W);          /* the row sums of all windows, then the column sums of all windows */
    g1_xyzz* cols = rows + 256ull * W;
    if (W < ROWCOL_PACKED_WINDOWS) {
        /* few windows: depth is the cost; cooperative sums and bit-wise weights */
        typedef CoopReduce<RowColSrc> RowCol;
        typedef CoopReduce<BitSumSrc> BitSum;
        typedef CoopReduce<GroupSumSrc> GroupSum;
        WS(bits, g1_xyzz, 16u * (uint32_t)W);
        WS(scaled, g1_xyzz, 16u * (uint32_t)W);
        RT((launch_coop<RowCol::BLOCK>(384u * (uint32_t)W, ctx->stream, RowCol{RowColSrc{bucket, rows, cols}})));
        RT((launch_coop<BitSum::BLOCK>(16u * (uint32_t)W, ctx->stream, BitSum{BitSumSrc{rows, cols, bits}})));
        RT((launch_coop<BitSumScale::BLOCK>((16u * (uint32_t)W + 63u) / 64u, ctx->stream, BitSumScale{bits, 16u * (uint32_t)W, scaled})));
        RT((launch_coop<GroupSum::BLOCK>((uint32_t)W, ctx->stream, GroupSum{GroupSumSrc{scaled, 16u, wsum}})));
        return TC_OK;
    }
    WS(w_rc, g1_xyzz, 2u * (uint32_t)W);     /* [0, W): columns, [W, 2W): rows */
    WS(s_rc, g1_xyzz, 2u * (uint32_t)W);
    {
        if ((uint64_t)W * 4096u > 0xFFFFFFF0ull) return fail(ctx, TC_ERR_SHAPE, "too many windows in one launch");
        WS(pieces, g1_xyzz, 4096ull * W);
        WS(redo, uint32_t, 4096ull * W + 1);
        RT(rt::launch<64>(1, ctx->stream, Fill32{redo, 0u}));
        BigRowColSums L1{bucket, 1, (uint32_t)W, pieces, redo, redo + 1};
        BigRowColSums L2{pieces, 2, (uint32_t)W, rows, redo, redo + 1};
        uint32_t redo_lanes = (uint32_t)std::min<uint64_t>(L1.lanes(), ACC_RESIDENT_LANES);
        RT((rt::launch_waves<64, 2>(L1.lanes(), ctx->stream, L1)));
        RT(rt::launch<64>(redo_lanes, ctx->stream, StridedRedo<BigRowColSums>{L1, redo_lanes}));
        RT(rt::launch<64>(1, ctx->stream, Fill32{redo, 0u}));
        RT((rt::launch_waves<64, 2>(L2.lanes(), ctx->stream, L2)));
        redo_lanes = (uint32_t)std::min<uint64_t>(L2.lanes(), ACC_RESIDENT_LANES);
        RT(rt::launch<64>(redo_lanes, ctx->stream, StridedRedo<BigRowColSums>{L2, redo_lanes}));
    }
    RT((launch_coop<256>(2u * (uint32_t)W, ctx->stream,
                         WeightedBlockSum<256>{cols, 256u * (uint32_t)W, w_rc, s_rc, rows, (uint32_t)W})));
    RT(rt::launch<64>((uint32_t)W, ctx->stream, RowColFinish{w_rc + W, s_rc + W, w_rc, wsum}));
    return TC_OK;
}

/* one launch for a list of jobs of the same kind (lanes[j] lanes for job j) */
template <int BLOCK, class F>
static int launch_jobs(tc_ctx* ctx, const std::vector<F>& jobs, const std::vector<uint64_t>& lanes) {
    if (jobs.empty()) return TC_OK;
    std::vector<uint64_t> first(jobs.size() + 1, 0);
    for (size_t j = 0; j < jobs.size(); ++j) first[j + 1] = first[j] + lanes[j];
    if (first.back() > 0xFFFFFFFFull) return fail(ctx, TC_ERR_SHAPE, "too many openings in one batch");
    if (!first.back()) return TC_OK;
    F* d_jobs = (F*)ws_alloc(ctx, sizeof(F) * jobs.size());
    uint64_t* d_first = ws_array<uint64_t>(ctx, first.size());
    if (!d_jobs || !d_first) return fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed");
    TRY(h2d(ctx, d_jobs, jobs.data(), sizeof(F) * jobs.size()));
    TRY(h2d(ctx, d_first, first.data(), sizeof(uint64_t) * first.size()));
    RT(rt::launch<BLOCK>(first.back(), ctx->stream, JobList<F>{d_jobs, d_first, (uint32_t)jobs.size()}));
    return TC_OK;
}

/* the scale and the quantised values of `count` fp16 tensors in five launches, whatever the count */
extern "C" int tc_encode_batch_scaled(tc_ctx* ctx, int count, const void* const* d_src, const size_t* n, float* d_inv_scale,
                                      void* const* d_dst) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (count < 0 || (count && (!d_src || !n || !d_inv_scale || !d_dst))) return fail(ctx, TC_ERR_ARG, "null argument");
        if ((uintptr_t)d_inv_scale & 3u) return fail(ctx, TC_ERR_ARG, "misaligned buffer");
        for (int i = 0; i < count; ++i) {
            if ((!d_src[i] || !d_dst[i]) && n[i]) return fail(ctx, TC_ERR_ARG, "null buffer");
            if (((uintptr_t)d_src[i] & 1u) || ((uintptr_t)d_dst[i] & 1u)) return fail(ctx, TC_ERR_ARG, "misaligned buffer");
            if (n[i] > 0xFFFFFFFFull) return fail(ctx, TC_ERR_SHAPE, "tensor too large");
        }
        if (!count) return TC_OK;
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        uint32_t* result = (uint32_t*)d_inv_scale;
        /* workgroups per tensor: together they fill the chip, and no tensor has more than its share of atomics */
        const uint32_t per_tensor = (uint32_t)std::max<uint64_t>(4, 2048 / (uint64_t)count);
        std::vector<AbsMaxF16> amax;
        std::vector<uint32_t> first(1, 0);
        std::vector<EncodeF16x8Strided> wide;
        std::vector<EncodeF16> narrow;
        std::vector<uint64_t> n_wide, n_narrow;
        for (int i = 0; i < count; ++i) {
            if (!n[i]) continue;
            uint32_t groups = (uint32_t)std::min<uint64_t>(std::min<uint32_t>(per_tensor, ABSMAX_MAX_GROUPS),
                                                           (n[i] / 8 + AbsMaxF16::BLOCK - 1) / AbsMaxF16::BLOCK);
            if (groups == 0) groups = 1;
            amax.push_back(AbsMaxF16{(const uint16_t*)d_src[i], (uint64_t)n[i], groups, result + i});
            first.push_back(first.back() + groups);
            bool aligned = (((uintptr_t)d_src[i] | (uintptr_t)d_dst[i]) & 15u) == 0;
            size_t bulk = aligned ? n[i] / 8 : 0;
            if (bulk) {
                uint32_t lanes = (uint32_t)((bulk + 7) / 8);          /* eight 16-byte pieces per lane */
                wide.push_back(EncodeF16x8Strided{EncodeF16x8{(const Words16*)d_src[i], (Words16*)d_dst[i], 0.0f, d_inv_scale + i}, (uint32_t)bulk, lanes});
                n_wide.push_back(lanes);
            }
            if (n[i] > 8 * bulk) {
                narrow.push_back(EncodeF16{(const uint16_t*)d_src[i] + 8 * bulk, (int16_t*)d_dst[i] + 8 * bulk, 0.0f, d_inv_scale + i});
                n_narrow.push_back(n[i] - 8 * bulk);
            }
        }
        RT(rt::launch<64>((uint32_t)count, ctx->stream, Fill32{result, 0u}));
        if (!amax.empty()) {
            WS(d_jobs, AbsMaxF16, amax.size());
            WS(d_first, uint32_t, first.size());
            TRY(h2d(ctx, d_jobs, amax.data(), sizeof(AbsMaxF16) * amax.size()));
            TRY(h2d(ctx, d_first, first.data(), sizeof(uint32_t) * first.size()));
            RT((launch_coop<AbsMaxF16Batch::BLOCK>(first.back(), ctx->stream, AbsMaxF16Batch{d_jobs, d_first, (uint32_t)amax.size()})));
        }
        RT(rt::launch<64>((uint32_t)count, ctx->stream, InvScaleFromAbsMax{result}));
        TRY((launch_jobs<256>(ctx, wide, n_wide)));
        TRY((launch_jobs<256>(ctx, narrow, n_narrow)));
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* plan of a call that may not allocate (tc_commit_static): entries per sub-run of the first pass and tiles of the
 * counting sort, chosen so that TC_STATIC_MAX_TERMS terms fit into TC_STATIC_SCRATCH_BYTES */
static const uint32_t STATIC_L1 = 16;
static const uint32_t STATIC_TILES = 16;

/* passes over partial sums with at least this many lanes fill the chip and take the kernels with the addition expanded
 * in place (and their second launch for the exceptional sums); smaller ones are bound by depth and launches */
#if defined(TC_HOST_EMU)
static const uint64_t FAST_PASS_LANES = 64;            /* the CPU build of the tests takes them from tiny sizes on */
#else
static const uint64_t FAST_PASS_LANES = 131072;
#endif
static const uint32_t MAX_ACC_PASSES = 8;
/* from this many sub-runs on, the accumulation takes them in the order of their lengths (three short launches) */
#if defined(TC_HOST_EMU)
static const uint64_t ORDERED_LANES_MIN = 64;
#else
static const uint64_t ORDERED_LANES_MIN = 1ull << 20;
#endif

/* from this many 16-bit terms on, a launch sorts them in two levels */
#if defined(TC_HOST_EMU)
static const uint64_t TWO_LEVEL_SORT_MIN = 64;
static const uint64_t SORT_SEVEN_BITS_MAX_TERMS = 4096;        /* the CPU build of the tests meets both word layouts */
static const uint64_t SORT_MIN_BIN_LOAD = 1;
#else
static const uint64_t TWO_LEVEL_SORT_MIN = 1ull << 23;
static const uint64_t SORT_SEVEN_BITS_MAX_TERMS = 1ull << 24;
/* ... and only where the bins hold a quarter of a tile on average: a batch of many small tensors would end up with a
 * workgroup and five barriers per handful of entries */
static const uint64_t SORT_MIN_BIN_LOAD = SORT_TILE / 4;
#endif

/* One MSM problem: result = sum_i [e(s_i)] pts[i] over n terms */
struct MsmProblem {
    const g1_affine* pts;
    const void* scalars;
    uint64_t n;
    const void* sub = nullptr;     /* DT_DIFF8 / DT_DIFF16: value = scalars[i] - sub[i] */
    uint32_t shift = 0;            /* DT_SPLIT16M: pts[i + shift] = 2^8 pts[i] */
};
/* digits per term: one per window, except where the digits of a term share a window */
static int msm_digits(int dtype, int W) { return dtype == DT_SPLIT16M ? 2 : W; }
static void msm_config(const tc_ctx* ctx, int dtype, uint64_t n, int* W, int* c) {
    if (dtype == TC_I8) { *W = 1; *c = 8; }
    else if (dtype == TC_I16) { *W = 1; *c = 16; }
    else if (dtype == DT_DIFF8 || dtype == DT_DIFF16) { *W = 2; *c = 9; }
    else if (dtype == DT_SPLIT16) { *W = 2; *c = 8; }
    else if (dtype == DT_SPLIT16M) { *W = 1; *c = 8; }
    else if (dtype == DT_FR128) { *W = 17; *c = 8; }
    else {
        *c = ctx->opt[TC_OPT_FR_WINDOW] ? (int)ctx->opt[TC_OPT_FR_WINDOW] : n >= 32768 ? 16 : 8;
        *W = 256 / *c;
    }
}
/* perm[lane] = sub-run (slot of the pass), longest first: the sub-runs of bucket b are the slots lstart[b] ..
 * lstart[b + 1] over its entries start[b] .. start[b + 1]; lstart = null: one slot per bucket.  `lanes` bounds the
 * number of slots from above. */
static int order_lanes(tc_ctx* ctx, const uint32_t* start, const uint32_t* lstart, uint32_t nbk, uint64_t lanes, uint32_t** out_perm) {
    uint32_t* perm = ws_array<uint32_t>(ctx, lanes);
    uint32_t* bins = ws_array<uint32_t>(ctx, 3 * SUBRUN_BINS);          /* histogram, bin starts, cursors */
    if (!perm || !bins) return fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed");
    RT(rt::launch<64>(SUBRUN_BINS, ctx->stream, Fill32{bins, 0u}));
    RT((launch_coop<SubrunHist::BLOCK>((nbk + SubrunHist::BLOCK - 1) / SubrunHist::BLOCK, ctx->stream, SubrunHist{start, lstart, nbk, bins})));
    RT(rt::launch<64>(1, ctx->stream, SubrunBinStarts{bins, bins + SUBRUN_BINS, bins + 2 * SUBRUN_BINS}));
    RT((launch_coop<SubrunOrder::BLOCK>((nbk + SubrunOrder::BLOCK - 1) / SubrunOrder::BLOCK, ctx->stream,
                                        SubrunOrder{start, lstart, nbk, bins + SUBRUN_BINS, bins + 2 * SUBRUN_BINS, perm})));
    *out_perm = perm;
    return TC_OK;
}

/* `count` problems of one scalar type and window plan, run through shared launches: the buckets of
 * problem p are the keys p * nbk .. (p + 1) * nbk of one big bucket space, so every pass (prefix
 * sums, balanced bucket sums, bucket reduction, window combination) is one launch for all problems. */
static int msm_engine_multi(tc_ctx* ctx, int count, const MsmProblem* prob, int dtype, int W, int c, g1_xyzz* results) {
    uint32_t nb = 1u << (c - 1);
    uint32_t nbk_pp = (uint32_t)W * nb;
    const int D = msm_digits(dtype, W);
    uint64_t items = 0, max_items = 0;
    for (int p = 0; p < count; ++p) {
        items += prob[p].n * (uint64_t)D;
        max_items = std::max<uint64_t>(max_items, prob[p].n * (uint64_t)D);
    }
    uint64_t nbk64 = (uint64_t)nbk_pp * (uint64_t)count;
    if (items > 0xFFFFFFF0ull || nbk64 > 0x7FFFFFFFull) return fail(ctx, TC_ERR_SHAPE, "MSM batch too large");
    uint32_t nbk = (uint32_t)nbk64;
    uint32_t nchunks = (nbk + SCAN_CHUNK - 1) / SCAN_CHUNK;

    WS(cnt, uint32_t, nbk);
    WS(cursor, uint32_t, nbk);
    WS(start, uint32_t, nbk + 1);
    WS(lstart, uint32_t, nbk + 1);
    WS(lstart2, uint32_t, nbk + 1);
    WS(tot_a, uint32_t, nchunks + 1);
    WS(tot_b, uint32_t, nchunks + 1);
    WS(tot_max, uint32_t, nchunks + 1);
    WS(sorted, uint32_t, items ? items : 1);
    WS(tables, const g1_affine*, (uint32_t)count);
    {
        const g1_affine* one = prob[0].pts;            /* a single problem needs no host array */
        std::vector<const g1_affine*> many;
        if (count > 1) {
            many.resize(count);
            for (int p = 0; p < count; ++p) many[p] = prob[p].pts;
        }
        TRY(upload_small(ctx, tables, count > 1 ? many.data() : &one, sizeof(void*) * (size_t)count));
    }

    /* Lanes of the first pass: sub-runs of at most L1 entries, about twice as many as the chip holds at once
     * (the accumulation kernel keeps 3 waves per SIMD), so that the second round evens out what the first left
     * uneven; at least 4 and at most 64 entries each.  Measured on the 2^21-entry int16 tensor: the kernel itself
     * is fastest with the shortest sub-runs (the first entry of a sub-run is a copy, not an addition), the later
     * passes with the longest, and steps in flight run equally fast from 4 to 13.  Not longer than half the
     * average bucket load either: longer sub-runs leave the lanes of a wave with very different amounts of work
     * (measured, with the 32-bit-limb accumulation of the time, on the 64 openings of the LLaMA2-7B-shaped forward, row buckets of 16 entries on average: sub-runs
     * of 8 and 16 entries 136 and 138 ms, of 24 and 32 entries 145 and 163 ms; on that forward's build, 101 entries
     * per bucket: sub-runs of 50 entries and one middle pass 69.2 ms, of 64 entries and no middle pass 70.3 ms). */
    const uint64_t target_lanes = 2 * ACC_RESIDENT_LANES;
    uint32_t L1 = (uint32_t)std::min<uint64_t>(64, std::max<uint64_t>(4, (items + target_lanes - 1) / target_lanes));
    /* (launches large enough to hand their sub-runs out in the order of their lengths need no such bound: with it
     * the LLaMA2-7B-shaped step takes 126.4 ms, with sub-runs of 64 entries 125.9 ms, and no less with 80 to 128) */
    if (ctx->static_mode || items / L1 + nbk + 1 < ORDERED_LANES_MIN)
        L1 = (uint32_t)std::min<uint64_t>(L1, std::max<uint64_t>(4, (items + 2 * (uint64_t)nbk - 1) / (2 * (uint64_t)nbk)));
    if (ctx->opt[TC_OPT_ACC_SUBRUN]) L1 = (uint32_t)ctx->opt[TC_OPT_ACC_SUBRUN];
    if (ctx->static_mode) L1 = STATIC_L1;      /* fewer, longer sub-runs: the partial sums must fit the static scratch */
    /* fan-in of the middle passes: with few buckets a pass costs the chain of additions of one lane, and shorter
     * chains in more passes win (flat commitment of 2^21 terms: 2.74 / 2.70 / 2.59 / 3.08 ms with 16 / 8 / 4 / 2) */
    const uint32_t L2 = ctx->opt[TC_OPT_ACC_FANIN] && !ctx->static_mode ? (uint32_t)ctx->opt[TC_OPT_ACC_FANIN] : nbk <= ScanSmall::MAX_N ? 4 : 16;

    uint32_t max_count = 0;        /* largest bucket: fixes how many shrinking passes are needed */
    if ((dtype != TC_FR && dtype != DT_FR128) || ((nbk_pp == 4096 || nbk_pp == 2176) && !ctx->static_mode)) {
        /* small scalars (one or two digits per term), and full-width scalars in 8-bit windows (4096 keys per problem):
         * tile histograms in LDS, no global atomics */
        /* tiles per problem: enough workgroups to fill the chip, but no tile so short that most of a workgroup's 1024
         * lanes (sixteen bytes of scalars per lane and step) find nothing to do -- the rows of a batch of openings,
         * tens of thousands of problems of a few thousand terms, are one tile each */
        uint64_t max_terms = 0;
        for (int p = 0; p < count; ++p) max_terms = std::max<uint64_t>(max_terms, prob[p].n);
        const uint64_t tile_terms_min = (dtype == TC_FR || dtype == DT_FR128) ? 1024 : 8192;      /* a full-width term is W digits' worth of work for its lane */
        uint32_t n_wg = (uint32_t)std::min<uint64_t>(256, std::max<uint64_t>(1, std::min<uint64_t>(4096 / (uint64_t)count, max_terms / tile_terms_min)));
        if (ctx->static_mode) n_wg = STATIC_TILES;     /* the tile histograms are n_wg rows of the key space */
        /* many 16-bit magnitudes: sorted by the upper key bits first, then by the lower ones, in tiles that a workgroup
         * sorts in LDS (the index of a term shares a word with its lower key bits on the way: seven of them for
         * problems of up to 2^24 terms, six up to 2^25) */
        bool two_level = nbk_pp == 32768 && dtype == TC_I16 && !ctx->static_mode && items >= TWO_LEVEL_SORT_MIN &&
                         max_terms <= 2 * SORT_SEVEN_BITS_MAX_TERMS;
        const uint32_t sort_low = max_terms <= SORT_SEVEN_BITS_MAX_TERMS ? 7u : 6u;
        for (int p = 0; p < count; ++p) two_level = two_level && !prob[p].sub;
        two_level = two_level && items / ((uint64_t)count * (32768u >> sort_low)) >= SORT_MIN_BIN_LOAD;
        if (two_level) {
            uint64_t tiles = (max_terms + SORT_TILE - 1) / SORT_TILE;
            if (tiles * (uint64_t)count <= (1ull << 20)) n_wg = (uint32_t)tiles;
            else two_level = false;
        }
        TileProblem one;
        std::vector<TileProblem> many;
        if (count > 1) many.resize(count);
        TileProblem* h_prob = count > 1 ? many.data() : &one;
        for (int p = 0; p < count; ++p) {
            memset((void*)&h_prob[p], 0, sizeof(TileProblem));
            h_prob[p].scalars = prob[p].scalars;
            h_prob[p].sub = prob[p].sub;
            h_prob[p].n = prob[p].n;
            /* a multiple of 16 terms, so that a tile of an aligned int8 / int16 array starts on a 16-byte boundary */
            h_prob[p].tile = (uint32_t)(((prob[p].n + n_wg - 1) / n_wg + 15) / 16 * 16);
            h_prob[p].shift = prob[p].shift;
        }
        WS(d_prob, TileProblem, (uint32_t)count);
        TRY(upload_small(ctx, d_prob, h_prob, sizeof(TileProblem) * (size_t)count));
        uint32_t groups = (uint32_t)count * n_wg;
        if (two_level) {
            const uint32_t bins_pp = 32768u >> sort_low, keys = 1u << sort_low;
            const uint32_t bins = (uint32_t)count * bins_pp;
            /* tiles of the second level: a bin of v entries has ceil(v / SORT_TILE) of them */
            const uint32_t max_tiles = (uint32_t)(items / SORT_TILE) + bins;
            WS(tile_bins, uint32_t, (uint64_t)groups * bins_pp);
            WS(bin_cnt, uint32_t, bins);
            WS(bin_start, uint32_t, bins + 1);
            WS(bin_tiles, uint32_t, bins + 1);
            WS(packed, uint32_t, items);
            WS(tile_keys, uint32_t, (uint64_t)max_tiles * keys);
            WS(tile_owner, uint32_t, max_tiles);
            RT((launch_coop<CountBins::BLOCK>(groups, ctx->stream, CountBins{d_prob, n_wg, sort_low, tile_bins})));
            RT(rt::launch<256>(bins, ctx->stream, TileColumnScan{bins_pp, n_wg, tile_bins, bin_cnt}));
            TRY(scan_counts(ctx, bin_cnt, bins, SORT_TILE, bin_start, bin_tiles, nullptr, tot_a, tot_b, tot_max));
            RT((launch_coop<ScatterBins::BLOCK>(groups, ctx->stream, ScatterBins{d_prob, n_wg, sort_low, tile_bins, bin_start, packed})));
            RT(rt::launch<256>(bins, ctx->stream, SortTileOwners{bin_tiles, tile_owner}));
            RT((launch_coop<CountKeys::BLOCK>(max_tiles, ctx->stream, CountKeys{packed, bin_start, bin_tiles, tile_owner, bins, sort_low, tile_keys})));
            RT(rt::launch<256>(nbk, ctx->stream, KeyColumnScan{bin_tiles, sort_low, tile_keys, cnt}));
            TRY(scan_counts(ctx, cnt, nbk, L1, start, lstart, nullptr, tot_a, tot_b, tot_max));
            RT(rt::memcpy_d2h(&max_count, tot_max + nchunks, 4, ctx->stream));
            RT((launch_coop<SortKeys::BLOCK>(max_tiles, ctx->stream, SortKeys{packed, bin_start, bin_tiles, tile_owner, bins, sort_low, tile_keys, start, sorted})));
        } else {
            WS(M, uint32_t, (uint64_t)count * n_wg * nbk_pp);
            /* counting tiles of a few thousand terms (the rows of a batch of openings) takes workgroups of 256 lanes: most of
             * 1024 would idle (0.53 -> 0.23 ms for the 23 552 rows of config 3's openings) */
            uint64_t max_tile = 0;
            for (int p = 0; p < count; ++p) max_tile = std::max<uint64_t>(max_tile, h_prob[p].tile);
            const bool narrow = nbk_pp == 128 && max_tile <= 16384 && !ctx->static_mode;
            if (narrow) RT((launch_coop<256>(groups, ctx->stream, CountTile<128, 256>{d_prob, dtype, D, c, n_wg, M})));
            else if (nbk_pp == 128) RT((launch_coop<1024>(groups, ctx->stream, CountTile<128>{d_prob, dtype, D, c, n_wg, M})));
            else if (nbk_pp == 256) RT((launch_coop<1024>(groups, ctx->stream, CountTile<256>{d_prob, dtype, D, c, n_wg, M})));
            else if (nbk_pp == 512) RT((launch_coop<1024>(groups, ctx->stream, CountTile<512>{d_prob, dtype, D, c, n_wg, M})));
            else if (nbk_pp == 4096) RT((launch_coop<1024>(groups, ctx->stream, CountTile<4096>{d_prob, dtype, D, c, n_wg, M})));
            else if (nbk_pp == 2176) RT((launch_coop<1024>(groups, ctx->stream, CountTile<2176>{d_prob, dtype, D, c, n_wg, M})));
            else if (nbk_pp == 32768) RT((launch_coop<1024>(groups, ctx->stream, CountTile<32768>{d_prob, dtype, D, c, n_wg, M})));
            else return fail(ctx, TC_ERR_STATE, "internal: unsupported key count");
            RT(rt::launch<256>(nbk, ctx->stream, TileColumnScan{nbk_pp, n_wg, M, cnt}));
            TRY(scan_counts(ctx, cnt, nbk, L1, start, lstart, nullptr, tot_a, tot_b, tot_max));
            if (!ctx->static_mode) RT(rt::memcpy_d2h(&max_count, tot_max + nchunks, 4, ctx->stream));
            /* (the scatter is faster with 1024 lanes even on short tiles: 1.04 against 1.28 ms on those rows) */
            if (nbk_pp == 128) RT((launch_coop<1024>(groups, ctx->stream, ScatterTile<128>{d_prob, dtype, D, c, n_wg, M, start, sorted})));
            else if (nbk_pp == 256) RT((launch_coop<1024>(groups, ctx->stream, ScatterTile<256>{d_prob, dtype, D, c, n_wg, M, start, sorted})));
            else if (nbk_pp == 512) RT((launch_coop<1024>(groups, ctx->stream, ScatterTile<512>{d_prob, dtype, D, c, n_wg, M, start, sorted})));
            else if (nbk_pp == 4096) RT((launch_coop<1024>(groups, ctx->stream, ScatterTile<4096>{d_prob, dtype, D, c, n_wg, M, start, sorted})));
            else if (nbk_pp == 2176) RT((launch_coop<1024>(groups, ctx->stream, ScatterTile<2176>{d_prob, dtype, D, c, n_wg, M, start, sorted})));
            else RT((launch_coop<1024>(groups, ctx->stream, ScatterTile<32768>{d_prob, dtype, D, c, n_wg, M, start, sorted})));
        }
    } else {
        if (ctx->static_mode) return fail(ctx, TC_ERR_STATE, "internal: full-width scalars in a call that may not allocate");
        RT(rt::launch<256>(nbk, ctx->stream, Fill32{cnt, 0u}));
        std::vector<MsmCount> j_count;
        std::vector<MsmScatter> j_scatter;
        std::vector<uint64_t> n_items;
        for (int p = 0; p < count; ++p) {
            j_count.push_back(MsmCount{prob[p].scalars, dtype, W, c, nb, cnt + (size_t)p * nbk_pp});
            j_scatter.push_back(MsmScatter{prob[p].scalars, dtype, W, c, nb, start + (size_t)p * nbk_pp, cursor + (size_t)p * nbk_pp, sorted});
            n_items.push_back(prob[p].n);
        }
        if (count == 1) RT(rt::launch<256>(prob[0].n, ctx->stream, j_count[0]));
        else TRY((launch_jobs<256>(ctx, j_count, n_items)));
        TRY(scan_counts(ctx, cnt, nbk, L1, start, lstart, cursor, tot_a, tot_b, tot_max));
        RT(rt::memcpy_d2h(&max_count, tot_max + nchunks, 4, ctx->stream));
        if (count == 1) RT(rt::launch<256>(prob[0].n, ctx->stream, j_scatter[0]));
        else TRY((launch_jobs<256>(ctx, j_scatter, n_items)));
    }

    uint64_t max_part = items / L1 + nbk + 1;          /* upper bound on first-pass lanes */
    WS(bufA, g1_xyzz, max_part);
    WS(bufB, g1_xyzz, max_part / L2 + nbk + 1);
    WS(bucket, g1_xyzz, nbk);
    WS(wsum, g1_xyzz, (uint64_t)W * count);
    /* lists of the lanes that a fast kernel gave up: [0] the count of the accumulation, [1 ..] which; the passes after
     * it have their counts in redo_pass and reuse the list (a pass starts when the one before is done) */
    WS(redo, uint32_t, max_part + 1);
    WS(redo_pass, uint32_t, MAX_ACC_PASSES);
    RT(rt::launch<64>(1, ctx->stream, Fill32{redo, 0u}));
    RT(rt::launch<64>(MAX_ACC_PASSES, ctx->stream, Fill32{redo_pass, 0u}));
    /* launches with many more lanes than the chip holds hand their sub-runs out in the order of their lengths */
    uint32_t* perm = nullptr;
    if (max_part >= ORDERED_LANES_MIN && !ctx->static_mode) TRY(order_lanes(ctx, start, lstart, nbk, max_part, &perm));
    {
        rt::event_t e0, e1;
        prof_begin(ctx, TC_PROF_BUCKET_ACC, &e0, &e1);
        int padded = 0;
        for (int p = 0; p < count; ++p) padded += table_is_padded(prob[p].pts) ? 1 : 0;
        if (padded == count) RT((rt::launch_waves<64, 3>(max_part, ctx->stream, AccAffine<TABLES_PADDED>{tables, nbk_pp, sorted, start, lstart, nbk, L1, bufA, redo, redo + 1, perm})));
        else if (padded == 0) RT((rt::launch_waves<64, 3>(max_part, ctx->stream, AccAffine<TABLES_PLAIN>{tables, nbk_pp, sorted, start, lstart, nbk, L1, bufA, redo, redo + 1, perm})));
        else RT((rt::launch_waves<64, 3>(max_part, ctx->stream, AccAffine<TABLES_MIXED>{tables, nbk_pp, sorted, start, lstart, nbk, L1, bufA, redo, redo + 1, perm})));
        prof_end(ctx, TC_PROF_BUCKET_ACC, e0, e1);
    }
    /* sub-runs with equal or opposite points in them: none in honest inputs; a degenerate input sends every sub-run
     * here, so the launch is as wide as the chip and its lanes stride over the list */
    {
        uint32_t redo_lanes = (uint32_t)std::min<uint64_t>(max_part, ACC_RESIDENT_LANES);
        RT(rt::launch<64>(redo_lanes, ctx->stream, AccAffineRedo{tables, nbk_pp, sorted, start, lstart, nbk, L1, bufA, redo, redo + 1, redo_lanes}));
    }

    /* Middle passes shrink the per-bucket partial count by L2 until at most L2 remain. */
    uint32_t acc_terms = 0, acc_lanes = 0;             /* non-zero digits and sub-runs of the first pass (profiling only) */
    if (ctx->profiling && !ctx->static_mode) {
        RT(rt::memcpy_d2h(&acc_terms, tot_a + nchunks, 4, ctx->stream));
        RT(rt::memcpy_d2h(&acc_lanes, tot_b + nchunks, 4, ctx->stream));
    }
    if (ctx->static_mode) {
        /* no wait for the stream: the passes are planned for the fullest bucket there could be, one that holds every
         * term of the largest problem (a pass over buckets that are already down to few partial sums copies them) */
        max_count = (uint32_t)max_items;
    } else {
        TRY(ctx_sync(ctx));
    }
    if (ctx->profiling && acc_terms >= acc_lanes) ctx->prof_units[TC_PROF_BUCKET_ACC] += acc_terms - acc_lanes;
    if (max_count > max_items) return fail(ctx, TC_ERR_STATE, "internal: bucket count exceeds the term count");
    uint64_t worst = ((uint64_t)max_count + L1 - 1) / L1;
    g1_xyzz *cur = bufA, *nxt = bufB;
    uint32_t *cur_start = lstart, *nxt_start = lstart2;
    uint64_t lanes_bound = max_part;
    /* (Leaving the middle passes out when the buckets outnumber the lanes the chip holds -- the last pass then
     * sums up to 64 partial sums per bucket -- was measured and is worse: its lanes diverge with the bucket loads;
     * 64 openings of the LLaMA2-7B-shaped forward 136 -> 206 ms, the build 69 -> 74 ms.) */
    uint32_t pass = 0;
    while (worst > L2) {
        /* counts of this pass = number of partials per bucket = differences of cur_start */
        RT(rt::launch<256>(nbk, ctx->stream, DiffCounts{cur_start, cnt}));
        TRY(scan_counts(ctx, cnt, nbk, L2, start, nxt_start, nullptr, tot_a, tot_b, tot_max));
        /* `start` now equals cur_start (prefix of the same counts) */
        lanes_bound = lanes_bound / L2 + nbk + 1;
        if (lanes_bound >= FAST_PASS_LANES && pass + 1 < MAX_ACC_PASSES) {
            uint32_t redo_lanes = (uint32_t)std::min<uint64_t>(lanes_bound, ACC_RESIDENT_LANES);
            uint32_t* pperm = nullptr;
            if (lanes_bound >= ORDERED_LANES_MIN && !ctx->static_mode) TRY(order_lanes(ctx, cur_start, nxt_start, nbk, lanes_bound, &pperm));
            RT((rt::launch_waves<64, 2>(lanes_bound, ctx->stream, AccXyzzFast{cur, cur_start, nxt_start, nbk, L2, nxt, redo_pass + pass, redo + 1, false, pperm})));
            RT(rt::launch<64>(redo_lanes, ctx->stream, AccXyzzRedo{cur, cur_start, nxt_start, nbk, L2, nxt, redo_pass + pass, redo + 1, false, redo_lanes}));
            ++pass;
        } else {
            RT(rt::launch<64>(lanes_bound, ctx->stream, AccXyzz{cur, cur_start, nxt_start, nbk, L2, nxt}));
        }
        std::swap(cur, nxt);
        std::swap(cur_start, nxt_start);
        worst = (worst + L2 - 1) / L2;
    }
    if (nbk >= FAST_PASS_LANES && nbk <= max_part) {
        uint32_t redo_lanes = (uint32_t)std::min<uint64_t>(nbk, ACC_RESIDENT_LANES);
        uint32_t* count = redo_pass + (MAX_ACC_PASSES - 1);
        uint32_t* pperm = nullptr;
        /* (after a middle pass nearly every bucket is down to one sum and the order is not worth its three launches) */
        if (nbk >= ORDERED_LANES_MIN && !ctx->static_mode && pass == 0) TRY(order_lanes(ctx, cur_start, nullptr, nbk, nbk, &pperm));
        RT((rt::launch_waves<64, 2>(nbk, ctx->stream, AccXyzzFast{cur, cur_start, nullptr, nbk, 0, bucket, count, redo + 1, true, pperm})));
        RT(rt::launch<64>(redo_lanes, ctx->stream, AccXyzzRedo{cur, cur_start, nullptr, nbk, 0, bucket, count, redo + 1, true, redo_lanes}));
    } else {
        RT(rt::launch<64>(nbk, ctx->stream, AccFinal{cur, cur_start, bucket}));
    }

    TRY(reduce_windows(ctx, bucket, W * count, nb, wsum));
    RT(rt::launch<64>((uint32_t)count, ctx->stream, WindowCombine{wsum, W, c, results}));
    return TC_OK;
}

/* result[0] = sum_i [e(s_i)] pts[i] */
static int msm_engine(tc_ctx* ctx, const g1_affine* pts, const void* d_scalars, int dtype, uint64_t n, g1_xyzz* result) {
    int W, c;
    msm_config(ctx, dtype, n, &W, &c);
    MsmProblem one{pts, d_scalars, n};
    return msm_engine_multi(ctx, 1, &one, dtype, W, c, result);
}

/* any list of problems: consecutive problems with the same scalar type and window plan share launches,
 * up to a bound on the batch size (the sorted index array is 4 bytes per term) */
static int msm_engine_list(tc_ctx* ctx, int count, const MsmProblem* prob, const int* dtype, g1_xyzz* results) {
    const uint64_t max_batch_items = 1ull << 30;
    const uint64_t max_batch_buckets = 1ull << 26;
    int i = 0;
    while (i < count) {
        int W, c;
        msm_config(ctx, dtype[i], prob[i].n, &W, &c);
        const int D = msm_digits(dtype[i], W);
        uint64_t items = prob[i].n * (uint64_t)D, buckets = (uint64_t)W << (c - 1);
        int j = i + 1;
        while (j < count) {
            int W2, c2;
            msm_config(ctx, dtype[j], prob[j].n, &W2, &c2);
            if (dtype[j] != dtype[i] || W2 != W || c2 != c) break;
            if (items + prob[j].n * (uint64_t)D > max_batch_items || buckets + ((uint64_t)W << (c - 1)) > max_batch_buckets) break;
            items += prob[j].n * (uint64_t)D;
            buckets += (uint64_t)W << (c - 1);
            ++j;
        }
        size_t mark = ctx->wsp->off;
        TRY(msm_engine_multi(ctx, j - i, prob + i, dtype[i], W, c, results + i));
        ctx->wsp->off = mark;            /* scratch is reusable by the next batch: the stream orders the kernels */
        i = j;
    }
    return TC_OK;
}

static int check_commit_args(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype) {
    if (!srs || !d_scalars) return fail(ctx, TC_ERR_ARG, "null argument");
    if (!valid_dtype_scalar(dtype)) return fail(ctx, TC_ERR_ARG, "unsupported scalar dtype");
    if (!srs->pts[0]) return fail(ctx, TC_ERR_STATE, "SRS has no points");
    return TC_OK;
}

extern "C" int tc_commit_batch(tc_ctx* ctx, int count, const tc_srs* const* srs, const void* const* d_scalars,
                               const int* dtype, uint8_t* out_g1) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (count < 0 || (count && (!srs || !d_scalars || !dtype || !out_g1))) return fail(ctx, TC_ERR_ARG, "null argument");
        for (int i = 0; i < count; ++i) TRY(check_commit_args(ctx, srs[i], d_scalars[i], dtype[i]));
        if (!count) return TC_OK;
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        WS(results, g1_xyzz, (uint32_t)count);
        std::vector<MsmProblem> prob(count);
        for (int i = 0; i < count; ++i) prob[i] = MsmProblem{srs_gather_table(srs[i], 0), d_scalars[i], srs[i]->n[0]};
        TRY(msm_engine_list(ctx, count, prob.data(), dtype, results));
        TRY(points_to_host(ctx, results, (uint32_t)count, out_g1));
        if (ctx->opt[TC_OPT_CHECK_LEVEL] >= 1) {
            for (int i = 0; i < count; ++i) {
                const uint8_t* b = out_g1 + 96 * (size_t)i;
                bool zero = true;
                for (int j = 0; j < 96; ++j) zero = zero && b[j] == 0;
                uint32_t w[24];
                memcpy(w, b, 96);
                if (!zero && !affine_on_curve(affine_from_canonical(w))) return fail(ctx, TC_ERR_STATE, "internal: a commitment is not on the curve");
            }
        }
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}
extern "C" int tc_commit(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype, uint8_t out_g1[96]) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!out_g1) return fail(ctx, TC_ERR_ARG, "null argument");
        return tc_commit_batch(ctx, 1, &srs, &d_scalars, &dtype, out_g1);
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* The commitment for callers that cannot allocate: the same kernels as tc_commit, every intermediate in the
 * device's static scratch array, the table pointer and the tile description sent as kernel arguments, the passes
 * over the partial sums planned from the term count alone (no value is read back, the stream is never waited for),
 * and the canonical bytes written to the caller's device buffer. */
struct StaticModeGuard {
    tc_ctx* ctx;
    explicit StaticModeGuard(tc_ctx* c) : ctx(c) {
        ctx->wsp = &ctx->ws_static;
        ctx->ws_static.off = 0;
        ctx->ws_static.demand = 0;
        ctx->static_mode = true;
    }
    ~StaticModeGuard() {
        ctx->wsp = &ctx->ws;
        ctx->static_mode = false;
    }
};
extern "C" int tc_commit_static(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype, void* d_out_g1) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!d_out_g1) return fail(ctx, TC_ERR_ARG, "null argument");
        if (((uintptr_t)d_out_g1 & 3u) != 0) return fail(ctx, TC_ERR_ARG, "the output buffer must be 4-byte aligned");
        TRY(check_commit_args(ctx, srs, d_scalars, dtype));
        if (dtype != TC_I8 && dtype != TC_I16) return fail(ctx, TC_ERR_ARG, "tc_commit_static takes int8 or int16 scalars");
        if (srs->n[0] > TC_STATIC_MAX_TERMS)
            return fail(ctx, TC_ERR_SHAPE, "tc_commit_static: the tensor has more than TC_STATIC_MAX_TERMS entries");
        if (!ctx->ws_static.base) return fail(ctx, TC_ERR_STATE, "static scratch not available");
        RT(rt::set_device(ctx->device));
        StaticModeGuard guard(ctx);
        WS(result, g1_xyzz, 1);
        WS(aff, g1_affine, 1);
        int W, c;
        msm_config(ctx, dtype, srs->n[0], &W, &c);
        MsmProblem one{srs_gather_table(srs, 0), d_scalars, srs->n[0]};
        TRY(msm_engine_multi(ctx, 1, &one, dtype, W, c, result));
        TRY(normalize(ctx, result, 1, aff));
        RT(rt::launch<64>(1, ctx->stream, ToCanonical{aff, (uint32_t*)d_out_g1}));
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}
extern "C" uint64_t tc_alloc_calls(void) { return rt::alloc_calls().load(); }

/* ======================================================================================= */
/* Open                                                                                    */
/* ======================================================================================= */
/* proof elements as XYZZ on the device (pi[0..m)), opened value as canonical Fr on the device */
/* One opening request: tensor, position. */
struct OpenSpec {
    const tc_srs* srs;
    const void* scalars;
    int dtype;
    uint32_t kappa[4];
    /* where the tensor's row commitments are kept between calls (a tree's slot for this leaf), or null: when the
     * slot is empty and the opening computes them, it leaves a device array of srs->shape[0] affine points there */
    g1_affine** row_cache = nullptr;
};

/* Openings of `count` tensors at once.  pi: count * 4 slots (m_i used), y: count values.
 * Every axis of every opening ends in full-width MSMs (quotient values against a suffix table, or the
 * row sums weighted by 1 / (zeta_k - zeta_kap)); all of them run through ONE list of problems so
 * that their window combinations (a chain of ~250 doublings each) proceed side by side.  Leading axes of
 * large small-integer tensors first go by rows, two 9-bit digits per entry, all rows of all openings in shared
 * launches.  Without the opening table: R_k = sum_t (T[k,t] - T[kap,t]) S[k,t] for every row k != kap, per opening.
 * With it (leading axis of the whole tensor, TC_SRS_OPEN_TABLE):
 *     pi_1 = sum_(k != kap) c_k A_k - sum_t T[kap,t] U[kap,t] + sum_t q[kap,t] S[kap,t],    c_k = 1 / (zeta_k - zeta_kap),
 * where the row commitments A_k = sum_t T[k,t] S[k,t] do not depend on the position: they are computed once per
 * tensor of the batch and kept in the caller's slot for later calls. */
/* full-width problems of fewer terms than this take 8-bit windows; those have their scalars halved (see below) */
static const uint64_t GLV_MAX_TERMS = 32768;
static int open_device_batch(tc_ctx* ctx, int count, const OpenSpec* spec, g1_xyzz* pi, fr_plain* y) {
    struct AxisJob {
        int open, axis;
        bool by_rows, use_table;
        uint64_t offset, inner, na;
        uint32_t d, kap;
        size_t row0;        /* first row problem (by_rows without the table) */
        int tensor;         /* index into `tensors` (use_table) */
        int small0;         /* the problem against row kap of the opening table (use_table) */
        int fr0;            /* first full-width problem */
    };
    struct TensorRows {     /* a tensor whose row commitments this batch needs */
        const tc_srs* srs;
        const void* scalars;
        g1_affine** slot;
        const g1_affine* rows;     /* d affine points once known */
        size_t row0;               /* first row problem when they are computed here */
        bool computed;
    };
    std::vector<AxisJob> jobs;
    std::vector<TensorRows> tensors;
    std::vector<FetchScalar> j_fetch;
    std::vector<MsmProblem> row_prob, small_prob;
    std::vector<int> row_dtype, small_dtype;
    for (int o = 0; o < count; ++o) {
        const tc_srs* srs = spec[o].srs;
        uint64_t offset = 0;
        for (int a = 0; a < srs->m; ++a) {
            AxisJob J;
            J.open = o; J.axis = a;
            J.na = srs->n[a]; J.d = srs->shape[a]; J.inner = J.na / J.d; J.kap = spec[o].kappa[a]; J.offset = offset;
            if (J.na > 0xFFFFFFFFull) return fail(ctx, TC_ERR_SHAPE, "slice too large");
            int dt = spec[o].dtype;
            J.by_rows = (dt == TC_I8 || dt == TC_I16) && J.d >= 2 && J.inner >= 2 && J.na >= 16384;
            J.use_table = J.by_rows && a == 0 && srs->open_tab != nullptr;
            J.row0 = row_prob.size(); J.fr0 = 0; J.tensor = -1; J.small0 = -1;
            size_t esz = dtype_size(dt);
            const uint8_t* base = (const uint8_t*)spec[o].scalars + offset * esz;
            int two_digits = dt == TC_I8 ? DT_DIFF8 : DT_DIFF16;
            /* plain rows of the tensor (the table's route) are one 8-bit digit (int8) or two (int16) per entry */
            int plain_digits = dt == TC_I8 ? TC_I8 : DT_SPLIT16;
            /* ... and with the shifted half of the table the two digits of a row share one window */
            int row_digits = dt == TC_I16 && srs->shifted && J.inner < 0x40000000ull ? DT_SPLIT16M : plain_digits;
            if (J.use_table) {
                for (size_t t = 0; t < tensors.size() && J.tensor < 0; ++t)
                    if (tensors[t].srs == srs && tensors[t].scalars == spec[o].scalars) J.tensor = (int)t;
                if (J.tensor < 0) {
                    TensorRows R{srs, spec[o].scalars, spec[o].row_cache, nullptr, row_prob.size(), false};
                    if (R.slot && *R.slot) {
                        R.rows = *R.slot;
                    } else {
                        R.computed = true;
                        for (uint32_t k = 0; k < J.d; ++k) {
                            MsmProblem P;
                            P.pts = srs_gather_table(srs, (uint64_t)k * J.inner);
                            P.scalars = base + (uint64_t)k * J.inner * esz;
                            P.n = J.inner;
                            P.shift = (uint32_t)srs->n[0];
                            row_prob.push_back(P);
                            row_dtype.push_back(row_digits);
                        }
                    }
                    J.tensor = (int)tensors.size();
                    tensors.push_back(R);
                } else if (!tensors[J.tensor].slot) {
                    tensors[J.tensor].slot = spec[o].row_cache;
                }
                MsmProblem P;            /* sum_t T[kap,t] U[kap,t] */
                P.pts = srs->open_tab + (uint64_t)J.kap * J.inner;
                P.scalars = base + (uint64_t)J.kap * J.inner * esz;
                P.n = J.inner;
                J.small0 = (int)small_prob.size();
                small_prob.push_back(P);
                small_dtype.push_back(plain_digits);
            } else if (J.by_rows) {
                for (uint32_t j = 0; j + 1 < J.d; ++j) {
                    uint32_t k = j < J.kap ? j : j + 1;
                    MsmProblem P;
                    P.pts = srs->pts[a] + (uint64_t)k * J.inner;
                    P.scalars = base + (uint64_t)k * J.inner * esz;
                    P.sub = base + (uint64_t)J.kap * J.inner * esz;
                    P.n = J.inner;
                    row_prob.push_back(P);
                    row_dtype.push_back(two_digits);
                }
            }
            jobs.push_back(J);
            offset += (uint64_t)J.kap * J.inner;
        }
        j_fetch.push_back(FetchScalar{spec[o].scalars, spec[o].dtype, offset, y + o});
    }
    TRY((launch_jobs<64>(ctx, j_fetch, std::vector<uint64_t>(j_fetch.size(), 1))));
    /* rows: all R_k of all openings, all A_k of the tensors that still lack them */
    g1_xyzz* Rk = nullptr;
    g1_affine* RkA = nullptr;
    if (!row_prob.empty()) {
        Rk = ws_array<g1_xyzz>(ctx, row_prob.size());
        RkA = ws_array<g1_affine>(ctx, row_prob.size());
        if (!Rk || !RkA) return fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed");
        TRY(msm_engine_list(ctx, (int)row_prob.size(), row_prob.data(), row_dtype.data(), Rk));
        TRY(normalize(ctx, Rk, row_prob.size(), RkA));
    }
    for (auto& R : tensors) {
        if (!R.computed) continue;
        R.rows = RkA + R.row0;
        if (R.slot && !*R.slot) {       /* keep them for later calls; without memory for that they are simply not kept */
            void* keep = nullptr;
            size_t bytes = (size_t)R.srs->shape[0] * sizeof(g1_affine);
            if (rt::dev_malloc(&keep, bytes) == 0) {
                RT(rt::memcpy_d2d(keep, R.rows, bytes, ctx->stream));
                *R.slot = (g1_affine*)keep;
            }
        }
    }
    /* the short problems against the opening table */
    g1_xyzz* res_small = nullptr;
    if (!small_prob.empty()) {
        res_small = ws_array<g1_xyzz>(ctx, small_prob.size());
        if (!res_small) return fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed");
        TRY(msm_engine_list(ctx, (int)small_prob.size(), small_prob.data(), small_dtype.data(), res_small));
    }
    /* full-width problems; the scalar work of all openings goes into six job lists, one launch each */
    std::vector<MsmProblem> fr_prob;
    std::vector<RowWeights> j_rw;
    std::vector<KappaWeights> j_kw;
    std::vector<KappaRowDirect> j_krd;
    std::vector<QuotientRows> j_qr;
    std::vector<QuotientKappaPartial> j_qkp;
    std::vector<QuotientKappaRow> j_qkr;
    std::vector<uint64_t> n_rw, n_kw, n_krd, n_qr, n_qkp, n_qkr;
    for (auto& J : jobs) {
        const tc_srs* srs = spec[J.open].srs;
        const void* sc = spec[J.open].scalars;
        int dt = spec[J.open].dtype;
        J.fr0 = (int)fr_prob.size();
        if (J.by_rows) {
            uint32_t rows = J.use_table ? J.d : J.d - 1;       /* with the table: every row, weight 0 at kap */
            WS(ck, fr_plain, rows);
            WS(wk, fr_t, J.d);
            WS(qk, fr_plain, J.inner);
            j_rw.push_back(RowWeights{srs->ax[J.axis], J.kap, J.use_table ? 1 : 0, ck});
            n_rw.push_back(rows);
            j_kw.push_back(KappaWeights{srs->ax[J.axis], J.kap, wk});
            n_kw.push_back(J.d);
            j_krd.push_back(KappaRowDirect{sc, dt, J.offset, J.d, J.kap, J.inner, srs->ax[J.axis], wk, qk});
            n_krd.push_back(J.inner);
            MsmProblem A, B;
            A.pts = J.use_table ? tensors[J.tensor].rows : RkA + J.row0; A.scalars = ck; A.n = rows;
            B.pts = srs->pts[J.axis] + (uint64_t)J.kap * J.inner; B.scalars = qk; B.n = J.inner;
            fr_prob.push_back(A);
            fr_prob.push_back(B);
        } else {
            WS(q, fr_plain, J.na);
            uint32_t chunks = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(256, 8192 / std::max<uint64_t>(J.inner, 1)));
            chunks = std::min<uint32_t>(chunks, J.d);
            WS(part, fr_t, (uint64_t)chunks * J.inner);
            j_qr.push_back(QuotientRows{sc, dt, J.offset, J.d, J.kap, J.inner, srs->ax[J.axis], q});
            n_qr.push_back(J.na);
            j_qkp.push_back(QuotientKappaPartial{J.d, J.kap, chunks, J.inner, srs->ax[J.axis], q, part});
            n_qkp.push_back((uint64_t)chunks * J.inner);
            j_qkr.push_back(QuotientKappaRow{J.kap, chunks, J.inner, srs->ax[J.axis], part, q});
            n_qkr.push_back(J.inner);
            MsmProblem A;
            A.pts = srs->pts[J.axis]; A.scalars = q; A.n = J.na;
            fr_prob.push_back(A);
        }
    }
    TRY((launch_jobs<64>(ctx, j_rw, n_rw)));
    TRY((launch_jobs<64>(ctx, j_kw, n_kw)));
    TRY((launch_jobs<64>(ctx, j_krd, n_krd)));
    TRY((launch_jobs<128>(ctx, j_qr, n_qr)));
    TRY((launch_jobs<128>(ctx, j_qkp, n_qkp)));
    TRY((launch_jobs<128>(ctx, j_qkr, n_qkr)));
    /* The short ones (8-bit windows) get their scalars halved with the endomorphism: twice the terms, 17 windows instead
     * of 32, and half the chain of doublings that combines the windows -- 248 doublings that two waves walk alone at
     * the end of the batch (64 openings of the LLaMA2-7B-shaped forward: 2.9 -> 1.5 ms).  The long ones (16-bit
     * windows, 32768 terms or more) stay as they are. */
    std::vector<int> fr_dtype(fr_prob.size(), TC_FR);
    {
        std::vector<GlvExpand> j_glv;
        std::vector<uint64_t> n_glv;
        for (size_t i = 0; i < fr_prob.size(); ++i) {
            MsmProblem& P = fr_prob[i];
            if (P.n == 0 || P.n >= GLV_MAX_TERMS) continue;
            WS(pts2, g1_affine, 2 * P.n);
            WS(k2, fr_plain, 2 * P.n);
            j_glv.push_back(GlvExpand{P.pts, (const fr_plain*)P.scalars, P.n, pts2, k2});
            n_glv.push_back(P.n);
            P.pts = pts2;
            P.scalars = k2;
            P.n *= 2;
            fr_dtype[i] = DT_FR128;
        }
        TRY((launch_jobs<64>(ctx, j_glv, n_glv)));
    }
    /* sort the full-width problems by window plan so that equal plans are neighbours and share launches */
    std::vector<int> order(fr_prob.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
    std::stable_sort(order.begin(), order.end(), [&](int x, int z) { return (fr_dtype[x] != DT_FR128) < (fr_dtype[z] != DT_FR128); });
    std::vector<MsmProblem> sorted_prob(fr_prob.size());
    std::vector<int> sorted_dtype(fr_prob.size(), TC_FR);
    for (size_t i = 0; i < order.size(); ++i) { sorted_prob[i] = fr_prob[order[i]]; sorted_dtype[i] = fr_dtype[order[i]]; }
    WS(res_sorted, g1_xyzz, fr_prob.size());
    TRY(msm_engine_list(ctx, (int)sorted_prob.size(), sorted_prob.data(), sorted_dtype.data(), res_sorted));
    std::vector<int32_t> where(fr_prob.size());           /* problem -> its place in the sorted results */
    for (size_t i = 0; i < order.size(); ++i) where[order[i]] = (int32_t)i;
    std::vector<CollectResult> j_out;
    for (auto& J : jobs)
        j_out.push_back(CollectResult{res_sorted, where[J.fr0], J.by_rows ? where[J.fr0 + 1] : -1, res_small, J.small0,
                                      pi + (size_t)J.open * 4 + J.axis});
    TRY((launch_jobs<64>(ctx, j_out, std::vector<uint64_t>(j_out.size(), 1))));
    return TC_OK;
}

static int open_device(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype, const uint32_t* kappa,
                       g1_xyzz* pi, fr_plain* y) {
    OpenSpec sp;
    sp.srs = srs; sp.scalars = d_scalars; sp.dtype = dtype;
    for (int a = 0; a < 4; ++a) sp.kappa[a] = a < srs->m ? kappa[a] : 0;
    WS(pi4, g1_xyzz, 4);
    TRY(open_device_batch(ctx, 1, &sp, pi4, y));
    RT(rt::memcpy_d2d(pi, pi4, sizeof(g1_xyzz) * (size_t)srs->m, ctx->stream));
    return TC_OK;
}

static int check_open_args(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype, const uint32_t* kappa) {
    TRY(check_commit_args(ctx, srs, d_scalars, dtype));
    if (!kappa) return fail(ctx, TC_ERR_ARG, "null argument");
    if (srs->flags & TC_SRS_MONOMIAL) return fail(ctx, TC_ERR_STATE, "openings need the Lagrange-basis SRS, this one is monomial");
    for (int a = 0; a < srs->m; ++a) {
        if (!srs->pts[a]) return fail(ctx, TC_ERR_STATE, "SRS was built without suffix tables");
        if (kappa[a] >= srs->shape[a]) return fail(ctx, TC_ERR_RANGE, "opening position outside the grid");
    }
    return TC_OK;
}

extern "C" int tc_open(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype, const uint32_t* kappa,
                       uint8_t out_y[32], uint8_t* out_pi) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!out_y || !out_pi) return fail(ctx, TC_ERR_ARG, "null argument");
        TRY(check_open_args(ctx, srs, d_scalars, dtype, kappa));
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        WS(pi, g1_xyzz, 4);
        WS(y, fr_plain, 1);
        TRY(open_device(ctx, srs, d_scalars, dtype, kappa, pi, y));
        RT(rt::memcpy_d2h(out_y, y, 32, ctx->stream));
        return points_to_host(ctx, pi, (uint32_t)srs->m, out_pi);
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ======================================================================================= */
/* Ver                                                                                     */
/* ======================================================================================= */
/* k = k2 * lambda + k1 with 0 <= k1 < lambda < 2^128 (k < r < lambda^2 + lambda + 1, so k2 < 2^128) */
static void glv_split(const uint32_t k[8], uint32_t k1[4], uint32_t k2[4]) { glv_split128(k, k1, k2); }
/* k = tau_i - (kappa + 1) mod r, split */
static void step_scalar(const tc_vk* vk, int i, uint32_t kappa, uint32_t k1[4], uint32_t k2[4]) {
    uint32_t w[8];
    memcpy(w, vk->tau[i], 32);
    fr_t k = fe_to_plain(fr_sub(fe_from_limbs<FrParams>(w), fe_from_u32<FrParams>(kappa + 1u)));
    glv_split(k.l, k1, k2);
}
extern "C" int tc_vk_from_trapdoor(const uint8_t* tau, int m, tc_vk** out) {
    try {
        if (!tau || !out || m < 1 || m > TC_MAX_ORDER) return TC_ERR_ARG;
        *out = nullptr;
        uint32_t w[8];
        for (int j = 0; j < m; ++j)
            if (!fr_bytes_canonical(tau + 32 * j, w)) return TC_ERR_RANGE;
        tc_vk* vk = new (std::nothrow) tc_vk();
        if (!vk) return TC_ERR_NOMEM;
        vk->m = m;
        memcpy(vk->tau, tau, 32 * (size_t)m);
        for (int i = 0; i < m; ++i)
            for (uint32_t kappa = 0; kappa < tc_vk::SPLIT_CACHE; ++kappa) step_scalar(vk, i, kappa, vk->k1[i][kappa], vk->k2[i][kappa]);
        *out = vk;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}
extern "C" void tc_vk_destroy(tc_vk* vk) { delete vk; }

/* fills the split scalars of a step: k_i = tau_i - (kappa_i + 1) mod r */
static void fill_step_scalars(const tc_vk* vk, const uint32_t* kappa, VerifyStep* st) {
    for (int i = 0; i < st->m; ++i) {
        if (kappa[i] < tc_vk::SPLIT_CACHE) {
            memcpy(st->k1[i], vk->k1[i][kappa[i]], 16);
            memcpy(st->k2[i], vk->k2[i][kappa[i]], 16);
        } else {
            step_scalar(vk, i, kappa[i], st->k1[i], st->k2[i]);
        }
    }
}

/* at most this many steps share the chain buffer (144 KiB per step) */
static const uint32_t VERIFY_CHUNK_STEPS = 4096;

/* runs the steps on the device; ok[i] = 1 iff step i verifies */
static int verify_steps(tc_ctx* ctx, const tc_vk* vk, const std::vector<VerifyStep>& steps, std::vector<uint32_t>& ok) {
    uint32_t n = (uint32_t)steps.size();
    ok.assign(n, 0);
    if (!n) return TC_OK;
    (void)vk;
    TRY(ensure_gtable(ctx));
    WS(d_steps, VerifyStep, n);
    WS(d_ok, uint32_t, n);
    uint32_t chunk = n < VERIFY_CHUNK_STEPS ? n : VERIFY_CHUNK_STEPS;
    WS(d_chain, g1_jac, (uint64_t)chunk * VERIFY_CHAINS * VERIFY_BITS);
    WS(d_part, g1_xyzz, (uint64_t)chunk * VERIFY_MAX_GROUPS);
    TRY(h2d(ctx, d_steps, steps.data(), sizeof(VerifyStep) * n));
    RT(rt::launch<256>(n, ctx->stream, Fill32{d_ok, 1u}));
    for (uint32_t c0 = 0; c0 < n; c0 += chunk) {       /* the chain buffer serves one chunk of steps after the other */
        uint32_t cn = n - c0 < chunk ? n - c0 : chunk;
        rt::event_t e0, e1;
        prof_begin(ctx, TC_PROF_VERIFY_CHAIN, &e0, &e1);
        int ce = launch_coop<VerifyChain::BLOCK>((VERIFY_CHAINS * cn + 63) / 64, ctx->stream, VerifyChain{d_steps + c0, VERIFY_CHAINS * cn, d_ok + c0, d_chain});
        prof_end(ctx, TC_PROF_VERIFY_CHAIN, e0, e1);
        RT(ce);
        int mmax = 1;
        for (uint32_t i = c0; i < c0 + cn; ++i) mmax = steps[i].m > mmax ? steps[i].m : mmax;
        uint32_t groups = (uint32_t)mmax + 1u;
        typedef CoopReduce<VerifyGroupSrc> Sum;
        typedef CoopReduce<VerifyDecideSrc> Decide;
        RT((launch_coop<Sum::BLOCK>(cn * groups, ctx->stream, Sum{VerifyGroupSrc{d_steps + c0, ctx->gtable, d_chain, d_ok + c0, groups, d_part}})));
        RT((launch_coop<Decide::BLOCK>(cn, ctx->stream, Decide{VerifyDecideSrc{d_part, groups, d_ok + c0}})));
    }
    RT(rt::memcpy_d2h(ok.data(), d_ok, 4ull * n, ctx->stream));
    TRY(ctx_sync(ctx));
    return TC_OK;
}

extern "C" int tc_verify(tc_ctx* ctx, const tc_vk* vk, int m, const uint32_t* shape, const uint8_t commitment[96],
                         const uint32_t* kappa, const uint8_t y[32], const uint8_t* pi) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!vk || !shape || !commitment || !kappa || !y || !pi) return fail(ctx, TC_ERR_ARG, "null argument");
        if (!shape_ok(m, shape, nullptr) || m > vk->m) return fail(ctx, TC_ERR_SHAPE, "bad shape");
        for (int j = 0; j < m; ++j)
            if (kappa[j] >= shape[j]) return fail(ctx, TC_ERR_RANGE, "opening position outside the grid");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        std::vector<VerifyStep> steps(1);
        memset(&steps[0], 0, sizeof(VerifyStep));
        memcpy(steps[0].C, commitment, 96);
        memcpy(steps[0].y, y, 32);
        for (int j = 0; j < m; ++j) memcpy(steps[0].pi[j], pi + 96 * j, 96);
        steps[0].m = m;
        fill_step_scalars(vk, kappa, &steps[0]);
        std::vector<uint32_t> ok;
        TRY(verify_steps(ctx, vk, steps, ok));
        if (!ok[0]) return fail(ctx, TC_ERR_VERIFY, "opening rejected");
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ======================================================================================= */
/* Terkle Tree                                                                             */
/* ======================================================================================= */
extern "C" void tc_tree_destroy(tc_tree* tree) {
    if (!tree) return;
    for (g1_affine* rows : tree->row_cache)
        if (rows) rt::dev_free(rows);
    if (tree->block) {
        TreePool* pool = tree->pool.get();
        if (pool && !pool->closed && tree->block_cap > pool->cap) {
            if (pool->block) rt::dev_free(pool->block);
            pool->block = tree->block;
            pool->cap = tree->block_cap;
        } else if (pool && !pool->closed && !pool->block) {
            pool->block = tree->block;
            pool->cap = tree->block_cap;
        } else {
            rt::dev_free(tree->block);
        }
    }
    delete tree;
}
extern "C" int tc_terkle_root(const tc_tree* tree, uint8_t out_g1[96]) {
    try {
        if (!tree || !out_g1) return TC_ERR_ARG;
        memcpy(out_g1, tree->root, 96);
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}
extern "C" int tc_terkle_levels(const tc_tree* tree) { return tree ? (int)tree->levels.size() : TC_ERR_ARG; }
extern "C" int tc_terkle_level_info(const tc_tree* tree, int level, uint32_t* grid, uint64_t* n_nodes) {
    try {
        if (!tree || level < 0 || level >= (int)tree->levels.size()) return TC_ERR_ARG;
        if (grid)
            for (int j = 0; j < tree->m; ++j) grid[j] = tree->levels[level].grid[j];
        if (n_nodes) *n_nodes = tree->levels[level].n;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}
extern "C" int tc_terkle_node(tc_ctx* ctx, const tc_tree* tree, int level, uint64_t index, uint8_t out_g1[96]) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!tree || !out_g1 || level < 0 || level >= (int)tree->levels.size()) return fail(ctx, TC_ERR_ARG, "bad argument");
        if (index >= tree->levels[level].n) return fail(ctx, TC_ERR_RANGE, "node index outside the level");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        return affine_to_host(ctx, tree->levels[level].C + index, 1, out_g1);
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

static TreeGeom make_geom(const tc_tree* t, const uint32_t* below, const uint32_t* grid) {
    TreeGeom g;
    g.m = t->m;
    g.B = t->B;
    for (int j = 0; j < 4; ++j) {
        g.node[j] = j < t->m ? t->node_shape[j] : 1;
        g.below[j] = j < t->m ? below[j] : 1;
        g.grid[j] = j < t->m ? grid[j] : 1;
    }
    return g;
}

/* gather the children of one node as a dense tensor of the node shape (zero padded) */
struct GatherNodeSmall {
    TreeGeom g;
    const void* payload;
    int dtype;
    uint64_t node;
    void* out;
    TC_DEV void operator()(uint32_t k) const {
        int64_t f = child_index(g, node, k);
        int32_t v = f < 0 ? 0 : small_scalar(payload, dtype, (uint64_t)f);
        if (dtype == DT_I8) ((int8_t*)out)[k] = (int8_t)v; else ((int16_t*)out)[k] = (int16_t)v;
    }
};
struct GatherNodeFr {
    TreeGeom g;
    const fr_plain* below;
    uint64_t node;
    fr_plain* out;
    TC_DEV void operator()(uint32_t k) const {
        int64_t f = child_index(g, node, k);
#pragma unroll
        for (int i = 0; i < 8; ++i) out[k].l[i] = f < 0 ? 0u : below[f].l[i];
    }
};

/* Checks a tree description and lays the tree out: level grids bottom-up and one device block for the commitments
 * and phi values of every level (taken from the context's pool when it is large enough).  Nothing is computed. */
static int tree_prepare(tc_ctx* ctx, const tc_tree_desc* desc, tc_tree** out) {
    *out = nullptr;
    uint64_t n_payload = 0, B = 0;
    if (!shape_ok(desc->m, desc->grid, &n_payload) || !shape_ok(desc->m, desc->node_shape, &B))
        return fail(ctx, TC_ERR_SHAPE, "bad grid or node shape");
    const tc_srs* ns = desc->node_srs;
    if (!ns) return fail(ctx, TC_ERR_ARG, "node SRS missing");
    if (ns->m != desc->m) return fail(ctx, TC_ERR_SHAPE, "node SRS order differs from the grid order");
    for (int j = 0; j < desc->m; ++j)
        if (ns->shape[j] != desc->node_shape[j]) return fail(ctx, TC_ERR_SHAPE, "node SRS shape differs from node_shape");
    if (ns->flags & TC_SRS_MONOMIAL) return fail(ctx, TC_ERR_STATE, "trees need the Lagrange-basis SRS, this one is monomial");
    bool more_than_one = false;
    for (int j = 0; j < desc->m; ++j) more_than_one = more_than_one || desc->node_shape[j] > 1;
    if (!more_than_one) return fail(ctx, TC_ERR_SHAPE, "node shape must have more than one entry");
    if (desc->leaf_kind == TC_LEAF_ENTRIES) {
        if (!desc->d_payload) return fail(ctx, TC_ERR_ARG, "payload missing");
        if (desc->dtype != TC_I8 && desc->dtype != TC_I16) return fail(ctx, TC_ERR_ARG, "payload must be int8 or int16");
    } else if (desc->leaf_kind == TC_LEAF_TENSORS) {
        if (!desc->leaf_srs || !desc->d_leaf_scalars || !desc->leaf_dtype) return fail(ctx, TC_ERR_ARG, "leaf arrays missing");
        for (uint64_t i = 0; i < n_payload; ++i) {
            TRY(check_commit_args(ctx, desc->leaf_srs[i], desc->d_leaf_scalars[i], desc->leaf_dtype[i]));
            if (desc->leaf_srs[i]->flags & TC_SRS_MONOMIAL) return fail(ctx, TC_ERR_STATE, "trees need the Lagrange-basis SRS, a leaf SRS is monomial");
        }
    } else {
        return fail(ctx, TC_ERR_ARG, "bad leaf kind");
    }
    RT(rt::set_device(ctx->device));
    TRY(ws_reset(ctx));

    tc_tree* t = new (std::nothrow) tc_tree();
    if (!t) return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    t->m = desc->m;
    t->B = (uint32_t)B;
    t->node_srs = ns;
    t->leaf_kind = desc->leaf_kind;
    t->d_payload = desc->d_payload;
    t->dtype = desc->dtype;
    for (int j = 0; j < desc->m; ++j) { t->grid[j] = desc->grid[j]; t->node_shape[j] = desc->node_shape[j]; }
    if (desc->leaf_kind == TC_LEAF_TENSORS) {
        t->leaf_srs.assign(desc->leaf_srs, desc->leaf_srs + n_payload);
        t->leaf_scalars.assign(desc->d_leaf_scalars, desc->d_leaf_scalars + n_payload);
        t->leaf_dtype.assign(desc->leaf_dtype, desc->leaf_dtype + n_payload);
        t->row_cache.assign(n_payload, nullptr);
    }
    /* level grids, bottom-up */
    {
        uint32_t g[4] = {1, 1, 1, 1};
        for (int j = 0; j < t->m; ++j) g[j] = t->grid[j];
        bool first = true;
        for (;;) {
            bool blocked = !(first && t->leaf_kind == TC_LEAF_TENSORS);
            TreeLevel lv;
            lv.n = 1;
            bool all_one = true;
            for (int j = 0; j < t->m; ++j) {
                lv.grid[j] = blocked ? (g[j] + t->node_shape[j] - 1) / t->node_shape[j] : g[j];
                lv.n *= lv.grid[j];
                all_one = all_one && lv.grid[j] == 1;
                g[j] = lv.grid[j];
            }
            t->levels.push_back(lv);
            first = false;
            if (all_one) break;
            if (t->levels.size() >= MAX_LEVELS) {
                delete t;
                return fail(ctx, TC_ERR_SHAPE, "tree too deep");
            }
        }
    }
    int rc = TC_OK;
    {
        size_t total = 0;
        for (auto& lv : t->levels) total += ((size_t)lv.n * sizeof(g1_affine) + 255) / 256 * 256 + ((size_t)lv.n * sizeof(fr_plain) + 255) / 256 * 256;
        t->pool = ctx->tree_pool;
        if (ctx->tree_pool->block && ctx->tree_pool->cap >= total) {
            t->block = ctx->tree_pool->block;
            t->block_cap = ctx->tree_pool->cap;
            ctx->tree_pool->block = nullptr;
            ctx->tree_pool->cap = 0;
        } else if (rt::dev_malloc(&t->block, total) == 0) {
            t->block_cap = total;
        } else {
            t->block = nullptr;
        }
        if (!t->block) {
            rc = fail(ctx, TC_ERR_NOMEM, "tree level allocation failed");
        } else {
            uint8_t* at = (uint8_t*)t->block;
            for (auto& lv : t->levels) {
                lv.C = (g1_affine*)at;
                at += ((size_t)lv.n * sizeof(g1_affine) + 255) / 256 * 256;
                lv.phi = (fr_plain*)at;
                at += ((size_t)lv.n * sizeof(fr_plain) + 255) / 256 * 256;
            }
        }
    }
    if (rc != TC_OK) {
        tc_tree_destroy(t);
        return rc;
    }
    *out = t;
    return TC_OK;
}

extern "C" int tc_terkle_build(tc_ctx* ctx, const tc_tree_desc* desc, tc_tree** out) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!desc || !out) return fail(ctx, TC_ERR_ARG, "null argument");
        tc_tree* t = nullptr;
        TRY(tree_prepare(ctx, desc, &t));
        const tc_srs* ns = t->node_srs;
        int rc = TC_OK;
        bool use_fb = ns->fb[0] != nullptr;
        for (size_t L = 0; L < t->levels.size() && rc == TC_OK; ++L) {
            TreeLevel& lv = t->levels[L];
            size_t mark = ctx->wsp->off;
            do {
                if (lv.n > 0xFFFFFFFFull / t->B) { rc = fail(ctx, TC_ERR_SHAPE, "level too large"); break; }
                g1_xyzz* acc = ws_array<g1_xyzz>(ctx, lv.n);
                if (!acc) { rc = fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed"); break; }
                if (L == 0 && t->leaf_kind == TC_LEAF_TENSORS) {
                    std::vector<MsmProblem> prob(lv.n);
                    for (uint64_t i = 0; i < lv.n; ++i) prob[i] = MsmProblem{srs_gather_table(t->leaf_srs[i], 0), t->leaf_scalars[i], t->leaf_srs[i]->n[0]};
                    rc = msm_engine_list(ctx, (int)lv.n, prob.data(), t->leaf_dtype.data(), acc);
                } else {
                    const uint32_t* below = L == 0 ? t->grid : t->levels[L - 1].grid;
                    TreeGeom g = make_geom(t, below, lv.grid);
                    bool bottom = (L == 0);
                    if (use_fb) {
                        int e;
                        if (bottom && lv.n <= COOP_LEVEL_NODES) {
                            typedef CoopReduce<NodeSmallSrc> Sum;
                            e = launch_coop<Sum::BLOCK>((uint32_t)lv.n, ctx->stream, Sum{NodeSmallSrc{g, t->d_payload, t->dtype, ns->fb[0], acc}});
                        } else if (bottom) {
                            rt::event_t e0, e1;
                            prof_begin(ctx, TC_PROF_NODE_COMMIT, &e0, &e1);
                            e = rt::launch<64>(lv.n, ctx->stream, NodeCommitSmall{g, t->d_payload, t->dtype, ns->fb[0], acc});
                            prof_end(ctx, TC_PROF_NODE_COMMIT, e0, e1);
                        } else if (lv.n <= COOP_LEVEL_NODES) {
                            rt::event_t e0, e1;
                            prof_begin(ctx, TC_PROF_NODE_COMMIT_UPPER, &e0, &e1);
                            /* very few nodes: every (child, window) term its own lane, sums shared by four waves */
                            typedef CoopReduce<NodeWindowSrc> Sum;
                            e = launch_coop<Sum::BLOCK>((uint32_t)lv.n, ctx->stream, Sum{NodeWindowSrc{g, t->levels[L - 1].phi, ns->fb[0], acc}});
                            prof_end(ctx, TC_PROF_NODE_COMMIT_UPPER, e0, e1);
                        } else if ((t->B & (t->B - 1)) == 0 && t->B <= 64) {
                            int logB = 0;
                            while ((1u << logB) < t->B) ++logB;
                            /* few nodes: one lane's depth is the cost, spread the windows of a child over lanes too */
                            int logH = 0;
                            while (logB + logH < 6 && (2 << logH) <= FB_W && (lv.n << (logB + logH + 1)) <= SPLIT_LEVEL_LANES) ++logH;
                            uint64_t lanes = lv.n << (logB + logH);
                            rt::event_t e0, e1;
                            prof_begin(ctx, TC_PROF_NODE_COMMIT_UPPER, &e0, &e1);
                            if (logH == 0)      /* a level large enough to fill the chip: throughput counts */
                                e = launch_coop<256>((uint32_t)((lanes + 255) / 256), ctx->stream,
                                                     NodeCommitFrCoop<256>{g, t->levels[L - 1].phi, ns->fb[0], lv.n, logB, logH, acc});
                            else
                                e = launch_coop<64>((uint32_t)((lanes + 63) / 64), ctx->stream,
                                                    NodeCommitFrCoop<64>{g, t->levels[L - 1].phi, ns->fb[0], lv.n, logB, logH, acc});
                            prof_end(ctx, TC_PROF_NODE_COMMIT_UPPER, e0, e1);
                        } else {
                            g1_xyzz* part = ws_array<g1_xyzz>(ctx, lv.n * t->B);
                            if (!part) { rc = fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed"); break; }
                            e = rt::launch<64>(lv.n * t->B, ctx->stream, NodeCommitFr{g, t->levels[L - 1].phi, ns->fb[0], part});
                            if (!e) e = rt::launch<64>(lv.n, ctx->stream, SumGroups{part, t->B, acc});
                        }
                        if (e) { rc = fail_hip(ctx, e, "node commit"); break; }
                    } else {
                        /* large node shapes: every node is its own MSM over the gathered children */
                        size_t esz = bottom ? dtype_size(t->dtype) : 32;
                        void* z = ws_alloc(ctx, (size_t)t->B * esz);
                        if (!z) { rc = fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed"); break; }
                        for (uint64_t a = 0; a < lv.n && rc == TC_OK; ++a) {
                            int e = bottom ? rt::launch<64>(t->B, ctx->stream, GatherNodeSmall{g, t->d_payload, t->dtype, a, z})
                                           : rt::launch<64>(t->B, ctx->stream, GatherNodeFr{g, t->levels[L - 1].phi, a, (fr_plain*)z});
                            if (e) { rc = fail_hip(ctx, e, "gather"); break; }
                            size_t mk = ctx->wsp->off;
                            rc = msm_engine(ctx, ns->pts[0], z, bottom ? t->dtype : TC_FR, t->B, acc + a);
                            ctx->wsp->off = mk;
                        }
                        if (rc) break;
                    }
                }
                if (rc) break;
                rc = normalize(ctx, acc, lv.n, lv.C);
                if (rc) break;
                int e = rt::launch<64>(lv.n, ctx->stream, PhiKernel{lv.C, lv.phi});
                if (e) rc = fail_hip(ctx, e, "phi");
            } while (0);
            ctx->wsp->off = mark;
        }
        if (rc == TC_OK) rc = affine_to_host(ctx, t->levels.back().C, 1, t->root);
        if (rc != TC_OK) {
            rt::stream_sync(ctx->stream);
            tc_tree_destroy(t);
            return rc;
        }
        *out = t;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ---- a tree as a flat file: the commitments of every node, so that openings can be served by a later process ----
 * Header (little-endian), then the levels bottom-up, each the canonical 96-byte commitments of its nodes, row-major
 * in the level's grid:
 *     0  char[8]  "TCTREE\0\0"
 *     8  u32      format version (1)
 *    12  u32      curve (1 = BLS12-381, commitments in G1)
 *    16  u32      m
 *    20  u32[4]   payload grid (unused axes 1)
 *    36  u32[4]   node shape
 *    52  u32      leaf kind (TC_LEAF_ENTRIES / TC_LEAF_TENSORS)
 *    56  u32      number of levels
 *    60  u32      reserved (0)
 *    64  u64      number of commitments that follow (all levels)
 *    72  ...      commitments */
static const char TREE_MAGIC[8] = {'T', 'C', 'T', 'R', 'E', 'E', 0, 0};
static const size_t TREE_HEADER_BYTES = 72;

extern "C" int tc_terkle_export(tc_ctx* ctx, const tc_tree* tree, void* host_buf, size_t* len) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!tree || !len) return fail(ctx, TC_ERR_ARG, "null argument");
        uint64_t count = 0;
        for (auto& lv : tree->levels) count += lv.n;
        size_t need = TREE_HEADER_BYTES + 96 * (size_t)count;
        size_t cap = *len;
        *len = need;
        if (!host_buf) return TC_OK;                /* size query */
        if (cap < need) return fail(ctx, TC_ERR_ARG, "buffer too small for the tree (needed size returned in *len)");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        uint8_t* o = (uint8_t*)host_buf;
        memset(o, 0, TREE_HEADER_BYTES);
        memcpy(o, TREE_MAGIC, 8);
        put_u32(o + 8, FILE_VERSION);
        put_u32(o + 12, CURVE_BLS12_381_G1);
        put_u32(o + 16, (uint32_t)tree->m);
        for (int j = 0; j < 4; ++j) {
            put_u32(o + 20 + 4 * j, j < tree->m ? tree->grid[j] : 1u);
            put_u32(o + 36 + 4 * j, j < tree->m ? tree->node_shape[j] : 1u);
        }
        put_u32(o + 52, (uint32_t)tree->leaf_kind);
        put_u32(o + 56, (uint32_t)tree->levels.size());
        put_u64(o + 64, count);
        o += TREE_HEADER_BYTES;
        for (auto& lv : tree->levels) {
            TRY(export_points(ctx, lv.C, lv.n, o));
            o += 96 * (size_t)lv.n;
        }
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

extern "C" int tc_terkle_import(tc_ctx* ctx, const tc_tree_desc* desc, const void* host_buf, size_t len, tc_tree** out) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!desc || !host_buf || !out) return fail(ctx, TC_ERR_ARG, "null argument");
        *out = nullptr;
        const uint8_t* in = (const uint8_t*)host_buf;
        if (len < TREE_HEADER_BYTES) return fail(ctx, TC_ERR_ARG, "tree file truncated: no complete header");
        if (memcmp(in, TREE_MAGIC, 8) != 0) return fail(ctx, TC_ERR_ARG, "not a tree file");
        if (get_u32(in + 8) != FILE_VERSION) return fail(ctx, TC_ERR_ARG, "unknown tree file version");
        if (get_u32(in + 12) != CURVE_BLS12_381_G1) return fail(ctx, TC_ERR_ARG, "the tree file is for another curve");
        tc_tree* t = nullptr;
        TRY(tree_prepare(ctx, desc, &t));
        int rc = TC_OK;
        do {
            bool same = get_u32(in + 16) == (uint32_t)t->m && get_u32(in + 52) == (uint32_t)t->leaf_kind &&
                        get_u32(in + 56) == (uint32_t)t->levels.size();
            for (int j = 0; j < 4 && same; ++j)
                same = get_u32(in + 20 + 4 * j) == (j < t->m ? t->grid[j] : 1u) &&
                       get_u32(in + 36 + 4 * j) == (j < t->m ? t->node_shape[j] : 1u);
            if (!same) { rc = fail(ctx, TC_ERR_SHAPE, "the tree file was written for another grid, node shape or leaf kind"); break; }
            uint64_t count = 0;
            for (auto& lv : t->levels) count += lv.n;
            if (get_u64(in + 64) != count) { rc = fail(ctx, TC_ERR_ARG, "node count in the tree file does not match its shape"); break; }
            if (len != TREE_HEADER_BYTES + 96 * (size_t)count) { rc = fail(ctx, TC_ERR_ARG, "tree file truncated or too long for its node count"); break; }
            const uint8_t* src = in + TREE_HEADER_BYTES;
            for (auto& lv : t->levels) {
                rc = import_points(ctx, src, lv.n, lv.C);
                if (rc) break;
                int e = rt::launch<64>(lv.n, ctx->stream, PhiKernel{lv.C, lv.phi});
                if (e) { rc = fail_hip(ctx, e, "phi"); break; }
                src += 96 * (size_t)lv.n;
            }
            if (rc) break;
            rc = affine_to_host(ctx, t->levels.back().C, 1, t->root);
        } while (0);
        if (rc != TC_OK) {
            rt::stream_sync(ctx->stream);
            tc_tree_destroy(t);
            return rc;
        }
        *out = t;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ---- paths ------------------------------------------------------------------------------ */
extern "C" int tc_path_from_grid(int m, const uint32_t* grid, const uint32_t* node_shape, int leaf_kind,
                                 const uint32_t* leaf_index, int inner_m, const uint32_t* inner_shape,
                                 const uint32_t* inner_index, tc_path* out) {
    try {
        if (!grid || !node_shape || !leaf_index || !out) return TC_ERR_ARG;
        if (!shape_ok(m, grid, nullptr) || !shape_ok(m, node_shape, nullptr)) return TC_ERR_SHAPE;
        if (leaf_kind != TC_LEAF_ENTRIES && leaf_kind != TC_LEAF_TENSORS) return TC_ERR_ARG;
        bool grow = false;
        for (int j = 0; j < m; ++j) {
            if (leaf_index[j] >= grid[j]) return TC_ERR_RANGE;
            grow = grow || node_shape[j] > 1;
        }
        if (!grow) return TC_ERR_SHAPE;
        /* bottom-up, then reversed */
        uint32_t pos[4] = {0, 0, 0, 0}, g[4] = {1, 1, 1, 1};
        for (int j = 0; j < m; ++j) { pos[j] = leaf_index[j]; g[j] = grid[j]; }
        std::vector<std::vector<uint32_t>> kap;
        bool first = true;
        for (;;) {
            bool blocked = !(first && leaf_kind == TC_LEAF_TENSORS);
            bool all_one = true;
            if (blocked) {
                std::vector<uint32_t> k(4, 0);
                for (int j = 0; j < m; ++j) {
                    k[j] = pos[j] % node_shape[j];
                    pos[j] /= node_shape[j];
                    g[j] = (g[j] + node_shape[j] - 1) / node_shape[j];
                }
                kap.push_back(k);
            }
            for (int j = 0; j < m; ++j) all_one = all_one && g[j] == 1;
            first = false;
            if (all_one) break;
            if (kap.size() >= TC_MAX_STEPS - 1) return TC_ERR_SHAPE;
        }
        memset(out, 0, sizeof *out);
        int s = 0;
        for (size_t i = kap.size(); i-- > 0; ++s) {
            out->m[s] = m;
            for (int j = 0; j < m; ++j) { out->shape[s][j] = node_shape[j]; out->kappa[s][j] = kap[i][j]; }
        }
        if (leaf_kind == TC_LEAF_TENSORS) {
            if (!inner_shape || !inner_index || !shape_ok(inner_m, inner_shape, nullptr)) return TC_ERR_ARG;
            out->m[s] = inner_m;
            for (int j = 0; j < inner_m; ++j) {
                if (inner_index[j] >= inner_shape[j]) return TC_ERR_RANGE;
                out->shape[s][j] = inner_shape[j];
                out->kappa[s][j] = inner_index[j];
            }
            ++s;
        }
        out->n_steps = s;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}

static uint64_t flat_of(const uint32_t* idx, const uint32_t* grid, int m) {
    uint64_t f = 0;
    for (int j = 0; j < m; ++j) f = f * grid[j] + idx[j];
    return f;
}

extern "C" int tc_terkle_open_batch(tc_ctx* ctx, const tc_tree* t, int count, const uint32_t* leaf_index,
                                    const uint32_t* inner_index, void* proof_buf, size_t proof_stride, size_t* proof_len) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!t || count < 0 || (count && (!leaf_index || !proof_buf || !proof_len))) return fail(ctx, TC_ERR_ARG, "null argument");
        if (t->leaf_kind == TC_LEAF_TENSORS && count && !inner_index) return fail(ctx, TC_ERR_ARG, "inner index missing");
        if (!count) return TC_OK;
        const tc_srs* ns = t->node_srs;
        int m = t->m;
        for (int a = 0; a < m; ++a)
            if (!ns->pts[a]) return fail(ctx, TC_ERR_STATE, "node SRS was built without suffix tables");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));

        int first_blocked = t->leaf_kind == TC_LEAF_TENSORS ? 1 : 0;
        int n_blocked = (int)t->levels.size() - first_blocked;
        bool use_fb = ns->fb[0] != nullptr;
        for (int a = 0; a < m && use_fb; ++a) use_fb = ns->fb[a] != nullptr;

        /* per path: node index and kappa at every blocked level (bottom-up), leaf flat index */
        struct PathInfo { std::vector<uint64_t> node; std::vector<std::vector<uint32_t>> kap; uint64_t leaf_flat; const uint32_t* inner; };
        std::vector<PathInfo> P(count);
        const uint32_t* inner_cursor = inner_index;
        for (int i = 0; i < count; ++i) {
            const uint32_t* li = leaf_index + (size_t)i * m;
            for (int j = 0; j < m; ++j)
                if (li[j] >= t->grid[j]) return fail(ctx, TC_ERR_RANGE, "leaf index outside the grid");
            uint32_t pos[4] = {0, 0, 0, 0};
            for (int j = 0; j < m; ++j) pos[j] = li[j];
            P[i].leaf_flat = flat_of(pos, t->grid, m);
            for (int b = 0; b < n_blocked; ++b) {
                std::vector<uint32_t> k(4, 0);
                for (int j = 0; j < m; ++j) { k[j] = pos[j] % t->node_shape[j]; pos[j] /= t->node_shape[j]; }
                P[i].node.push_back(flat_of(pos, t->levels[first_blocked + b].grid, m));
                P[i].kap.push_back(k);
            }
            if (t->leaf_kind == TC_LEAF_TENSORS) {
                const tc_srs* ls = t->leaf_srs[P[i].leaf_flat];
                for (int a = 0; a < ls->m; ++a) {
                    if (!ls->pts[a]) return fail(ctx, TC_ERR_STATE, "leaf SRS was built without suffix tables");
                    if (inner_cursor[a] >= ls->shape[a]) return fail(ctx, TC_ERR_RANGE, "inner index outside the leaf tensor");
                }
                P[i].inner = inner_cursor;
                inner_cursor += ls->m;
            }
        }
        /* proof sizes */
        std::vector<size_t> need(count);
        for (int i = 0; i < count; ++i) {
            size_t bytes = (size_t)n_blocked * (96 * (size_t)m + 32 + 96);
            if (t->leaf_kind == TC_LEAF_TENSORS) bytes += 96 * (size_t)t->leaf_srs[P[i].leaf_flat]->m + 32;
            else bytes -= 96;                               /* the bottom step carries no child commitment */
            need[i] = bytes;
            proof_len[i] = bytes;
            if (bytes > proof_stride) return fail(ctx, TC_ERR_ARG, "proof buffer too small");
        }

        /* blocked levels: pi and y for every (path, level) */
        uint32_t jobs = (uint32_t)count * (uint32_t)n_blocked;
        std::vector<uint8_t> h_pi((size_t)jobs * m * 96), h_y((size_t)jobs * 32);
        if (jobs) {
            WS(d_pi, g1_xyzz, (uint64_t)jobs * m);
            WS(d_y, fr_plain, jobs);
            if (use_fb) {
                NodeOpenTerms k;
                memset((void*)&k, 0, sizeof k);
                k.node.m = m;
                uint32_t terms = 0;
                for (int j = 0; j < 4; ++j) k.node.d[j] = j < m ? t->node_shape[j] : 1;
                for (int a = 0; a < m; ++a) {
                    k.axis_first[a] = terms;
                    terms += (uint32_t)ns->n[a];
                    k.ax[a] = ns->ax[a];
                    k.table[a] = ns->fb[a];
                }
                for (int a = m; a <= 4; ++a) k.axis_first[a] = terms;
                k.terms_per_job = terms;
                for (int b = 0; b < n_blocked; ++b) {
                    int L = first_blocked + b;
                    const uint32_t* below = L == 0 ? t->grid : t->levels[L - 1].grid;
                    k.lv[b].g = make_geom(t, below, t->levels[L].grid);
                    k.lv[b].payload = L == 0 ? t->d_payload : nullptr;
                    k.lv[b].dtype = t->dtype;
                    k.lv[b].below = L == 0 ? nullptr : t->levels[L - 1].phi;
                }
                std::vector<NodeOpenJob> hj(jobs);
                std::vector<uint32_t> seg((size_t)jobs * m + 1);
                for (int i = 0; i < count; ++i)
                    for (int b = 0; b < n_blocked; ++b) {
                        uint32_t j = (uint32_t)i * n_blocked + b;
                        hj[j].node = P[i].node[b];
                        for (int a = 0; a < 4; ++a) hj[j].kappa[a] = P[i].kap[b][a];
                        hj[j].level = b;
                        hj[j].term0 = j * terms;
                        for (int a = 0; a < m; ++a) seg[(size_t)j * m + a] = j * terms + k.axis_first[a];
                    }
                seg[(size_t)jobs * m] = jobs * terms;
                WS(d_jobs, NodeOpenJob, jobs);
                WS(d_seg, uint32_t, (uint64_t)jobs * m + 1);
                int logH = 0;
                while ((2u << logH) < (uint32_t)FB_W) ++logH;
                if ((((uint64_t)jobs * terms) << logH) > 0xFFFFFFFFull) return fail(ctx, TC_ERR_ARG, "too many openings in one batch");
                WS(d_terms, g1_xyzz, ((uint64_t)jobs * terms) << logH);
                TRY(h2d(ctx, d_jobs, hj.data(), sizeof(NodeOpenJob) * jobs));
                TRY(h2d(ctx, d_seg, seg.data(), 4 * seg.size()));
                k.jobs = d_jobs;
                k.out = d_terms;
                k.y_out = d_y;
                k.logH = logH;
                RT(rt::launch<64>(((uint64_t)jobs * terms) << logH, ctx->stream, k));
                typedef CoopReduce<SegmentSrc> Sum;
                RT((launch_coop<Sum::BLOCK>(jobs * (uint32_t)m, ctx->stream, Sum{SegmentSrc{d_terms, d_seg, 1u << logH, d_pi}})));
            } else {
                /* large node shapes: gather the node tensor and open it like any tensor */
                for (int i = 0; i < count; ++i)
                    for (int b = 0; b < n_blocked; ++b) {
                        int L = first_blocked + b;
                        uint32_t j = (uint32_t)i * n_blocked + b;
                        const uint32_t* below = L == 0 ? t->grid : t->levels[L - 1].grid;
                        TreeGeom g = make_geom(t, below, t->levels[L].grid);
                        size_t mk = ctx->wsp->off;
                        bool bottom = L == 0;
                        void* z = ws_alloc(ctx, (size_t)t->B * (bottom ? dtype_size(t->dtype) : 32));
                        if (!z) return fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed");
                        if (bottom) RT(rt::launch<64>(t->B, ctx->stream, GatherNodeSmall{g, t->d_payload, t->dtype, P[i].node[b], z}));
                        else RT(rt::launch<64>(t->B, ctx->stream, GatherNodeFr{g, t->levels[L - 1].phi, P[i].node[b], (fr_plain*)z}));
                        uint32_t kap[4];
                        for (int a = 0; a < 4; ++a) kap[a] = P[i].kap[b][a];
                        TRY(open_device(ctx, ns, z, bottom ? t->dtype : TC_FR, kap, d_pi + (uint64_t)j * m, d_y + j));
                        ctx->wsp->off = mk;
                    }
            }
            RT(rt::memcpy_d2h(h_y.data(), d_y, 32ull * jobs, ctx->stream));
            TRY(points_to_host(ctx, d_pi, jobs * (uint32_t)m, h_pi.data()));
        }
        /* leaf tensors: all openings in one batch */
        std::vector<std::vector<uint8_t>> leaf_part(count);
        if (t->leaf_kind == TC_LEAF_TENSORS) {
            std::vector<OpenSpec> specs(count);
            for (int i = 0; i < count; ++i) {
                const tc_srs* ls = t->leaf_srs[P[i].leaf_flat];
                specs[i].srs = ls;
                specs[i].scalars = t->leaf_scalars[P[i].leaf_flat];
                specs[i].dtype = t->leaf_dtype[P[i].leaf_flat];
                for (int a = 0; a < 4; ++a) specs[i].kappa[a] = a < ls->m ? P[i].inner[a] : 0;
            }
            WS(pi, g1_xyzz, 4ull * count);
            WS(y, fr_plain, (uint32_t)count);
            RT(rt::launch<64>(4ull * count, ctx->stream, FillIdentity{pi}));     /* slots of unused axes */
            TRY(open_device_batch(ctx, count, specs.data(), pi, y));
            std::vector<uint8_t> hy(32ull * count), hp(96ull * 4 * count);
            RT(rt::memcpy_d2h(hy.data(), y, 32ull * count, ctx->stream));
            TRY(points_to_host(ctx, pi, 4u * (uint32_t)count, hp.data()));
            for (int i = 0; i < count; ++i) {
                int lm = specs[i].srs->m;
                leaf_part[i].resize(96 * (size_t)lm + 32);
                memcpy(leaf_part[i].data(), hp.data() + 96ull * 4 * i, 96 * (size_t)lm);
                memcpy(leaf_part[i].data() + 96 * (size_t)lm, hy.data() + 32ull * i, 32);
            }
        }
        /* child commitments along the paths */
        uint32_t n_child = 0;
        std::vector<uint8_t> h_child;
        {
            /* for blocked level b (0 = lowest blocked) the child is the node of the level below on the path */
            std::vector<std::pair<int, uint64_t>> want;     /* (level, node) */
            for (int i = 0; i < count; ++i)
                for (int b = 0; b < n_blocked; ++b) {
                    int L = first_blocked + b;
                    if (L == 0) continue;
                    uint64_t child = (b == 0) ? P[i].leaf_flat : P[i].node[b - 1];
                    want.push_back({L - 1, child});
                }
            n_child = (uint32_t)want.size();
            if (n_child) {
                std::vector<const g1_affine*> src(n_child);
                for (uint32_t w = 0; w < n_child; ++w) src[w] = t->levels[want[w].first].C + want[w].second;
                WS(d_src, const g1_affine*, n_child);
                WS(can, uint32_t, 24ull * n_child);
                TRY(h2d(ctx, d_src, src.data(), sizeof(const g1_affine*) * n_child));
                RT(rt::launch<64>(n_child, ctx->stream, ToCanonicalGather{d_src, can}));
                h_child.resize(96ull * n_child);
                RT(rt::memcpy_d2h(h_child.data(), can, 96ull * n_child, ctx->stream));
                TRY(ctx_sync(ctx));
            }
        }
        /* assemble, top level first */
        uint32_t child_cursor = 0;
        for (int i = 0; i < count; ++i) {
            uint8_t* dst = (uint8_t*)proof_buf + (size_t)i * proof_stride;
            /* children were queued bottom-up for this path */
            uint32_t n_child_i = 0;
            for (int b = 0; b < n_blocked; ++b)
                if (first_blocked + b > 0) ++n_child_i;
            for (int b = n_blocked - 1; b >= 0; --b) {
                uint32_t j = (uint32_t)i * n_blocked + b;
                memcpy(dst, h_pi.data() + (size_t)j * m * 96, 96 * (size_t)m);
                dst += 96 * (size_t)m;
                memcpy(dst, h_y.data() + 32 * (size_t)j, 32);
                dst += 32;
                if (first_blocked + b > 0) {
                    uint32_t slot = child_cursor + (uint32_t)(b - (first_blocked ? 0 : 1));
                    memcpy(dst, h_child.data() + 96ull * slot, 96);
                    dst += 96;
                }
            }
            child_cursor += n_child_i;
            if (t->leaf_kind == TC_LEAF_TENSORS) {
                memcpy(dst, leaf_part[i].data(), leaf_part[i].size());
                dst += leaf_part[i].size();
            }
            if ((size_t)(dst - ((uint8_t*)proof_buf + (size_t)i * proof_stride)) != need[i]) return fail(ctx, TC_ERR_STATE, "internal: proof size mismatch");
        }
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

extern "C" int tc_terkle_open(tc_ctx* ctx, const tc_tree* tree, const uint32_t* leaf_index, const uint32_t* inner_index,
                              void* proof_buf, size_t* proof_len) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!proof_len) return fail(ctx, TC_ERR_ARG, "null argument");
        size_t cap = *proof_len;
        return tc_terkle_open_batch(ctx, tree, 1, leaf_index, inner_index, proof_buf, cap, proof_len);
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ---- path verification --------------------------------------------------------------------- */
extern "C" int tc_verify_paths_batch(tc_ctx* ctx, const tc_vk* vk, int count, const tc_path* paths, const uint8_t* roots,
                                     const uint8_t* leaf_values, const void* proofs, size_t proof_stride,
                                     const size_t* proof_len, int* results) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!vk || count < 0 || (count && (!paths || !roots || !leaf_values || !proofs || !proof_len || !results)))
            return fail(ctx, TC_ERR_ARG, "null argument");
        if (!count) return TC_OK;
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        std::vector<VerifyStep> steps;
        std::vector<int> first_step(count + 1, 0);
        std::vector<uint8_t> malformed(count, 0);
        std::vector<std::vector<uint8_t>> child_bytes;        /* per step: commitment carried to the next step (or empty) */
        for (int i = 0; i < count; ++i) {
            const tc_path& p = paths[i];
            first_step[i] = (int)steps.size();
            const uint8_t* src = (const uint8_t*)proofs + (size_t)i * proof_stride;
            size_t expect = 0;
            bool bad = p.n_steps < 1 || p.n_steps > TC_MAX_STEPS;
            for (int s = 0; s < p.n_steps && !bad; ++s) {
                if (p.m[s] < 1 || p.m[s] > vk->m || !shape_ok(p.m[s], p.shape[s], nullptr)) bad = true;
                else {
                    for (int j = 0; j < p.m[s]; ++j) bad = bad || p.kappa[s][j] >= p.shape[s][j];
                    expect += 96 * (size_t)p.m[s] + 32 + (s + 1 < p.n_steps ? 96 : 0);
                }
            }
            if (bad || expect != proof_len[i]) {
                malformed[i] = 1;
                continue;
            }
            const uint8_t* carried = roots + 96 * (size_t)i;
            for (int s = 0; s < p.n_steps; ++s) {
                VerifyStep st;
                memset(&st, 0, sizeof st);
                st.m = p.m[s];
                memcpy(st.C, carried, 96);
                for (int j = 0; j < st.m; ++j) {
                    memcpy(st.pi[j], src, 96);
                    src += 96;
                }
                fill_step_scalars(vk, p.kappa[s], &st);
                memcpy(st.y, src, 32);
                src += 32;
                steps.push_back(st);
                if (s + 1 < p.n_steps) {
                    child_bytes.emplace_back(src, src + 96);
                    carried = src;
                    src += 96;
                } else {
                    child_bytes.emplace_back();
                }
            }
        }
        first_step[count] = (int)steps.size();
        std::vector<uint32_t> ok;
        TRY(verify_steps(ctx, vk, steps, ok));
        /* phi of every carried commitment, on the device */
        uint32_t ns = (uint32_t)steps.size();
        std::vector<uint8_t> h_phi(32ull * (ns ? ns : 1), 0);
        if (ns) {
            std::vector<uint32_t> pts(24ull * ns, 0);
            for (uint32_t s = 0; s < ns; ++s)
                if (!child_bytes[s].empty()) memcpy(&pts[24ull * s], child_bytes[s].data(), 96);
            WS(d_pts, uint32_t, 24ull * ns);
            WS(d_phi, fr_plain, ns);
            TRY(h2d(ctx, d_pts, pts.data(), 96ull * ns));
            RT(rt::launch<64>(ns, ctx->stream, PhiCanonical{d_pts, d_phi}));
            RT(rt::memcpy_d2h(h_phi.data(), d_phi, 32ull * ns, ctx->stream));
            TRY(ctx_sync(ctx));
        }
        for (int i = 0; i < count; ++i) {
            if (malformed[i]) { results[i] = TC_ERR_VERIFY; continue; }
            bool good = true;
            for (int s = first_step[i]; s < first_step[i + 1]; ++s) {
                good = good && ok[s];
                bool last = s + 1 == first_step[i + 1];
                const uint8_t* yb = (const uint8_t*)steps[s].y;
                if (last) good = good && memcmp(yb, leaf_values + 32 * (size_t)i, 32) == 0;
                else good = good && memcmp(yb, &h_phi[32ull * s], 32) == 0;
            }
            results[i] = good ? TC_OK : TC_ERR_VERIFY;
        }
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

extern "C" int tc_verify_path(tc_ctx* ctx, const tc_vk* vk, const tc_path* path, const uint8_t root[96],
                              const uint8_t leaf_value[32], const void* proof, size_t proof_len) {
    try {
        if (!ctx) return TC_ERR_ARG;
        int result = TC_ERR_VERIFY;
        int rc = tc_verify_paths_batch(ctx, vk, 1, path, root, leaf_value, proof, proof_len, &proof_len, &result);
        if (rc != TC_OK) return rc;
        if (result != TC_OK) return fail(ctx, TC_ERR_VERIFY, "path rejected");
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ---- incremental update --------------------------------------------------------------------- */
extern "C" int tc_terkle_update(tc_ctx* ctx, tc_tree* tree, const uint32_t* leaf_index, const uint32_t* inner_index,
                                int64_t delta) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!tree || !leaf_index) return fail(ctx, TC_ERR_ARG, "null argument");
        tc_tree* t = tree;
        if (delta >= (1ll << 32) || delta <= -(1ll << 32)) return fail(ctx, TC_ERR_RANGE, "delta too large");
        const tc_srs* ns = t->node_srs;
        if (!ns->fb[0]) return fail(ctx, TC_ERR_STATE, "updates need the fixed-base node SRS");
        int m = t->m;
        for (int j = 0; j < m; ++j)
            if (leaf_index[j] >= t->grid[j]) return fail(ctx, TC_ERR_RANGE, "leaf index outside the grid");
        bool tensors = t->leaf_kind == TC_LEAF_TENSORS;
        if (tensors && !inner_index) return fail(ctx, TC_ERR_ARG, "inner index missing");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        WS(d_dphi, fr_plain, 1);
        typedef CoopReduce<UpdatePathSrc> Upd;
        uint32_t pos[4] = {0, 0, 0, 0};
        for (int j = 0; j < m; ++j) pos[j] = leaf_index[j];
        int level = 0;
        int from_dphi = 0;
        if (tensors) {
            uint64_t leaf_flat = flat_of(pos, t->grid, m);
            const tc_srs* ls = t->leaf_srs[leaf_flat];
            uint64_t inner_flat = 0;
            for (int a = 0; a < ls->m; ++a) {
                if (inner_index[a] >= ls->shape[a]) return fail(ctx, TC_ERR_RANGE, "inner index outside the leaf tensor");
                inner_flat = inner_flat * ls->shape[a] + inner_index[a];
            }
            if (t->row_cache[leaf_flat]) {           /* the tensor changes: its kept row commitments no longer hold */
                TRY(ctx_sync(ctx));
                rt::dev_free(t->row_cache[leaf_flat]);
                t->row_cache[leaf_flat] = nullptr;
            }
            RT((launch_coop<Upd::BLOCK>(1, ctx->stream, Upd{UpdatePathSrc{t->levels[0].C, t->levels[0].phi, leaf_flat, nullptr, 0,
                                                                          ls->pts[0] + inner_flat, delta, 0, d_dphi}})));
            level = 1;
            from_dphi = 1;
        }
        for (; level < (int)t->levels.size(); ++level) {
            uint32_t k[4] = {0, 0, 0, 0};
            for (int j = 0; j < m; ++j) { k[j] = pos[j] % t->node_shape[j]; pos[j] /= t->node_shape[j]; }
            uint64_t a = flat_of(pos, t->levels[level].grid, m);
            uint32_t kf = (uint32_t)flat_of(k, t->node_shape, m);
            RT((launch_coop<Upd::BLOCK>(1, ctx->stream, Upd{UpdatePathSrc{t->levels[level].C, t->levels[level].phi, a, ns->fb[0], kf,
                                                                          nullptr, delta, from_dphi, d_dphi}})));
            from_dphi = 1;
        }
        return affine_to_host(ctx, t->levels.back().C, 1, t->root);
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ======================================================================================= */
/* The coefficient route: interpolation, Algorithm 1                                       */
/* ======================================================================================= */
static bool interp_shape_ok(int m, const uint32_t* shape, uint64_t* total) {
    if (m < 1 || m > TC_MAX_INTERP_ORDER || !shape) return false;
    uint64_t n = 1;
    for (int j = 0; j < m; ++j) {
        if (shape[j] == 0) return false;
        n *= shape[j];
        if (n > (1ull << 31) - 1) return false;
    }
    *total = n;
    return true;
}

extern "C" int tc_interpolate_form(tc_ctx* ctx, int m, const uint32_t* shape, const void* d_scalars, int dtype, int form,
                                   void* d_coeffs) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!d_scalars || !d_coeffs) return fail(ctx, TC_ERR_ARG, "null argument");
        if (!valid_dtype_scalar(dtype)) return fail(ctx, TC_ERR_ARG, "unsupported scalar dtype");
        if (form != TC_INTERP_NEWTON && form != TC_INTERP_GREGORY && form != TC_INTERP_BARYCENTRIC)
            return fail(ctx, TC_ERR_ARG, "unknown interpolation form");
        uint64_t n = 0;
        if (!interp_shape_ok(m, shape, &n)) return fail(ctx, TC_ERR_SHAPE, "bad shape");
        RT(rt::set_device(ctx->device));
        TRY(ws_reset(ctx));
        uint32_t dmax = 1;
        for (int j = 0; j < m; ++j) dmax = std::max(dmax, shape[j]);
        /* 1 / l, 1 / l! and zeta_k = k + 1 up to the longest axis */
        std::vector<fr_t> inv(dmax), zeta(dmax), inv_fact(dmax);
        for (uint32_t i = 0; i < dmax; ++i) {
            inv[i] = fe_from_u32<FrParams>(i ? i : 1);
            zeta[i] = fe_from_u32<FrParams>(i + 1);
        }
        fr_batch_inverse(inv);
        inv_fact[0] = fe_one<FrParams>();
        for (uint32_t i = 1; i < dmax; ++i) inv_fact[i] = fr_mul(inv_fact[i - 1], inv[i]);
        WS(d_inv, fr_t, dmax);
        WS(d_zeta, fr_t, dmax);
        WS(d_aux, fr_t, dmax);             /* 1 / l! (Gregory) or the weights beta of the current axis (barycentric) */
        TRY(h2d(ctx, d_inv, inv.data(), sizeof(fr_t) * dmax));
        TRY(h2d(ctx, d_zeta, zeta.data(), sizeof(fr_t) * dmax));
        if (form == TC_INTERP_GREGORY) TRY(h2d(ctx, d_aux, inv_fact.data(), sizeof(fr_t) * dmax));
        const int nbuf = form == TC_INTERP_BARYCENTRIC ? 5 : 3;
        fr_t* buf[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
        for (int i = 0; i < nbuf; ++i) {
            buf[i] = ws_array<fr_t>(ctx, n);
            if (!buf[i]) return fail(ctx, TC_ERR_NOMEM, "device workspace allocation failed");
        }
        RT(rt::launch<256>(n, ctx->stream, ScalarsToFr{d_scalars, dtype, buf[0]}));
        std::vector<fr_t> beta;
        uint64_t outer = 1;
        for (int j = 0; j < m; ++j) {
            uint32_t d = shape[j];
            uint64_t inner = n / (outer * d);
            uint64_t lines = outer * inner;
            uint32_t lines_per_wg = d >= (uint32_t)InterpAxis<false>::BLOCK ? 1u : (uint32_t)InterpAxis<false>::BLOCK / d;
            uint64_t groups = (lines + lines_per_wg - 1) / lines_per_wg;
            if (d > 1 && form == TC_INTERP_BARYCENTRIC) {
                /* beta_l = (-1)^(d-1-l) / (l! (d-1-l)!) on the nodes 1 .. d */
                beta.resize(d);
                for (uint32_t l = 0; l < d; ++l) {
                    beta[l] = fr_mul(inv_fact[l], inv_fact[d - 1 - l]);
                    if ((d - 1 - l) & 1u) beta[l] = fr_neg(beta[l]);
                }
                /* the previous axis' launch may still read its weights: the copy is ordered behind it on the stream */
                TRY(h2d(ctx, d_aux, beta.data(), sizeof(fr_t) * d));
                InterpAxisBarycentric k;
                k.w = buf[0]; k.p[0] = buf[1]; k.p[1] = buf[2]; k.mm[0] = buf[3]; k.mm[1] = buf[4];
                k.outer = outer; k.inner = inner; k.d = d; k.lines_per_wg = lines_per_wg;
                k.beta = d_aux; k.zeta = d_zeta;
                RT((launch_coop_n<InterpAxisBarycentric::BLOCK>((uint32_t)groups, ctx->stream, k, (int)(d + 1))));
                std::swap(buf[0], buf[1 + (d & 1u)]);
            } else if (d > 1) {
                if (form == TC_INTERP_GREGORY) {
                    InterpAxis<true> k;
                    k.buf[0] = buf[0]; k.buf[1] = buf[1]; k.buf[2] = buf[2];
                    k.outer = outer; k.inner = inner; k.d = d; k.lines_per_wg = lines_per_wg;
                    k.inv_int = d_inv; k.zeta = d_zeta; k.inv_fact = d_aux;
                    RT((launch_coop_n<InterpAxis<true>::BLOCK>((uint32_t)groups, ctx->stream, k, (int)(2 * d - 1))));
                } else {
                    InterpAxis<false> k;
                    k.buf[0] = buf[0]; k.buf[1] = buf[1]; k.buf[2] = buf[2];
                    k.outer = outer; k.inner = inner; k.d = d; k.lines_per_wg = lines_per_wg;
                    k.inv_int = d_inv; k.zeta = d_zeta; k.inv_fact = nullptr;
                    RT((launch_coop_n<InterpAxis<false>::BLOCK>((uint32_t)groups, ctx->stream, k, (int)(2 * d - 1))));
                }
                std::swap(buf[0], buf[interp_result_buffer(d)]);      /* the next axis reads what this one produced */
            }
            outer *= d;
        }
        RT(rt::launch<256>(n, ctx->stream, FrToPlain{buf[0], (fr_plain*)d_coeffs}));
        TRY(ctx_sync(ctx));
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

extern "C" int tc_interpolate(tc_ctx* ctx, int m, const uint32_t* shape, const void* d_scalars, int dtype, void* d_coeffs) {
    try {
        return tc_interpolate_form(ctx, m, shape, d_scalars, dtype, TC_INTERP_NEWTON, d_coeffs);
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

extern "C" int tc_divide_by_linear(tc_ctx* ctx, int m, const uint32_t* shape, const void* d_coeffs, int axis,
                                   uint32_t kappa_axis, void* d_quotient, void* d_remainder) {
    try {
        if (!ctx) return TC_ERR_ARG;
        if (!d_coeffs || !d_quotient || !d_remainder) return fail(ctx, TC_ERR_ARG, "null argument");
        if (d_quotient == d_coeffs || d_remainder == d_coeffs || d_quotient == d_remainder) return fail(ctx, TC_ERR_ARG, "arrays may not alias");
        uint64_t n = 0;
        if (!interp_shape_ok(m, shape, &n)) return fail(ctx, TC_ERR_SHAPE, "bad shape");
        if (axis < 0 || axis >= m) return fail(ctx, TC_ERR_ARG, "axis outside the shape");
        if (kappa_axis >= shape[axis]) return fail(ctx, TC_ERR_RANGE, "position outside the grid");
        RT(rt::set_device(ctx->device));
        uint64_t outer = 1;
        for (int j = 0; j < axis; ++j) outer *= shape[j];
        uint32_t d = shape[axis];
        uint64_t inner = n / (outer * d);
        /* everything off the axis' degree 0 in r, and the whole of q, is written by the kernel; lines = outer * inner */
        RT(rt::launch<64>(outer * inner, ctx->stream,
                          DivideAxis{(const fr_plain*)d_coeffs, outer, inner, d, kappa_axis + 1u, (fr_plain*)d_quotient, (fr_plain*)d_remainder}));
        TRY(ctx_sync(ctx));
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return fail(ctx, TC_ERR_NOMEM, "host allocation failed");
    } catch (...) {
        return fail(ctx, TC_ERR_STATE, "internal: unexpected exception");
    }
}

/* ======================================================================================= */
/* Public verification with the pairing: host only                                         */
/* ======================================================================================= */
struct tc_vkp {
    int m = 0;
    pairing::g2_affine tau_h[TC_MAX_ORDER];
};

extern "C" int tc_vkp_from_trapdoor(const uint8_t* tau, int m, tc_vkp** out) {
    try {
        if (!tau || !out || m < 1 || m > TC_MAX_ORDER) return TC_ERR_ARG;
        *out = nullptr;
        tc_vkp* vkp = new (std::nothrow) tc_vkp();
        if (!vkp) return TC_ERR_NOMEM;
        vkp->m = m;
        pairing::g2_affine h = pairing::g2_generator();
        for (int j = 0; j < m; ++j) {
            uint32_t w[8];
            if (!fr_bytes_canonical(tau + 32 * j, w)) {
                delete vkp;
                return TC_ERR_RANGE;
            }
            vkp->tau_h[j] = pairing::g2_mul(w, 256, h);
        }
        *out = vkp;
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}
extern "C" void tc_vkp_destroy(tc_vkp* vkp) { delete vkp; }
extern "C" int tc_vkp_get(const tc_vkp* vkp, int axis, uint8_t out_g2[192]) {
    try {
        if (!vkp || !out_g2 || axis < -1 || axis >= vkp->m) return TC_ERR_ARG;
        pairing::g2_to_bytes(axis < 0 ? pairing::g2_generator() : vkp->tau_h[axis], out_g2);
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}

/* canonical bytes -> affine point on E; false when not canonical or not on the curve */
static bool g1_from_bytes_checked(const uint8_t* b, g1_affine* out) {
    uint32_t w[24];
    memcpy(w, b, 96);
    if (!canonical_fp(w) || !canonical_fp(w + 12)) return false;
    *out = affine_from_canonical(w);
    return affine_on_curve(*out);
}

extern "C" int tc_pairing(const uint8_t p_g1[96], const uint8_t q_g2[192], uint8_t out_gt[576]) {
    try {
        if (!p_g1 || !q_g2 || !out_gt) return TC_ERR_ARG;
        pairing::pair_t pr;
        if (!g1_from_bytes_checked(p_g1, &pr.p) || !pairing::g2_from_bytes(q_g2, &pr.q)) return TC_ERR_RANGE;
        pairing::gt_to_bytes(pairing::pairing_product({pr}), out_gt);
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}

/* Every opening's equation, moved to fixed second arguments,
 *     e(C - [y]G + sum_i [zeta_i] pi_i, H) prod_i e(-pi_i, [tau_i]H) = 1,
 * is raised to a weight rho and multiplied into one running equation: by bilinearity the weights go to the G1
 * side, so any number of openings costs m + 1 Miller loops and one final exponentiation.  The first opening has
 * weight 1, the others 128-bit weights drawn at random: a set of openings with a wrong one passes only with
 * probability about 2^-128. */
struct PairingBatch {
    g1_xyzz h_term = xyzz_identity();
    g1_xyzz tau_term[TC_MAX_ORDER];
    int m_used = 0;
    int count = 0;
    std::mt19937_64 rng{std::random_device{}()};
    PairingBatch() {
        for (int i = 0; i < TC_MAX_ORDER; ++i) tau_term[i] = xyzz_identity();
    }
};
static g1_xyzz weigh(const g1_xyzz& p, const uint32_t rho[4], bool unit) {
    if (unit) return p;
    return xyzz_mul_affine(rho, 128, xyzz_to_affine(p));
}
/* adds one opening; false when a point or the value is malformed */
static bool pairing_batch_add(PairingBatch* B, int m, const uint8_t* commitment, const uint32_t* kappa, const uint8_t* y,
                              const uint8_t* pi) {
    g1_affine C;
    uint32_t yw[8];
    if (!g1_from_bytes_checked(commitment, &C) || !fr_bytes_canonical(y, yw)) return false;
    bool unit = B->count == 0;
    uint32_t rho[4] = {1, 0, 0, 0};
    if (!unit)
        for (int i = 0; i < 4; ++i) rho[i] = (uint32_t)B->rng();
    g1_xyzz t = xyzz_add(xyzz_from_affine(C), xyzz_neg(xyzz_mul_affine(yw, 256, affine_generator())));
    for (int i = 0; i < m; ++i) {
        g1_affine p;
        if (!g1_from_bytes_checked(pi + 96 * (size_t)i, &p)) return false;
        uint32_t zeta[1] = {kappa[i] + 1u};
        t = xyzz_add(t, xyzz_mul_affine(zeta, 32, p));
        B->tau_term[i] = xyzz_add(B->tau_term[i], weigh(xyzz_from_affine(affine_neg(p)), rho, unit));
    }
    B->h_term = xyzz_add(B->h_term, weigh(t, rho, unit));
    if (m > B->m_used) B->m_used = m;
    ++B->count;
    return true;
}
static bool pairing_batch_check(const tc_vkp* vkp, const PairingBatch& B) {
    std::vector<pairing::pair_t> pairs;
    pairs.push_back({xyzz_to_affine(B.h_term), pairing::g2_generator()});
    for (int i = 0; i < B.m_used; ++i) pairs.push_back({xyzz_to_affine(B.tau_term[i]), vkp->tau_h[i]});
    return pairing::pairing_product_is_one(pairs);
}

extern "C" int tc_verify_pairing(const tc_vkp* vkp, int m, const uint32_t* shape, const uint8_t commitment[96],
                                 const uint32_t* kappa, const uint8_t y[32], const uint8_t* pi) {
    try {
        if (!vkp || !shape || !commitment || !kappa || !y || !pi) return TC_ERR_ARG;
        if (!shape_ok(m, shape, nullptr) || m > vkp->m) return TC_ERR_SHAPE;
        for (int j = 0; j < m; ++j)
            if (kappa[j] >= shape[j]) return TC_ERR_RANGE;
        PairingBatch B;
        if (!pairing_batch_add(&B, m, commitment, kappa, y, pi)) return TC_ERR_VERIFY;
        return pairing_batch_check(vkp, B) ? TC_OK : TC_ERR_VERIFY;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}

/* the structural checks and phi links of one path; its openings go into B.  false = reject */
static bool pairing_path_add(const tc_vkp* vkp, PairingBatch* B, const tc_path& p, const uint8_t* root,
                             const uint8_t* leaf_value, const uint8_t* proof, size_t proof_len) {
    if (p.n_steps < 1 || p.n_steps > TC_MAX_STEPS) return false;
    size_t expect = 0;
    for (int s = 0; s < p.n_steps; ++s) {
        if (p.m[s] < 1 || p.m[s] > vkp->m || !shape_ok(p.m[s], p.shape[s], nullptr)) return false;
        for (int j = 0; j < p.m[s]; ++j)
            if (p.kappa[s][j] >= p.shape[s][j]) return false;
        expect += 96 * (size_t)p.m[s] + 32 + (s + 1 < p.n_steps ? 96 : 0);
    }
    if (expect != proof_len) return false;
    const uint8_t* src = proof;
    const uint8_t* carried = root;
    for (int s = 0; s < p.n_steps; ++s) {
        const uint8_t* pi = src;
        const uint8_t* y = src + 96 * (size_t)p.m[s];
        src = y + 32;
        if (!pairing_batch_add(B, p.m[s], carried, p.kappa[s], y, pi)) return false;
        if (s + 1 < p.n_steps) {
            /* the opened value is phi of the commitment carried to the next step */
            g1_affine child;
            if (!g1_from_bytes_checked(src, &child)) return false;
            fr_t v = phi_map(child);
            if (memcmp(v.l, y, 32) != 0) return false;
            carried = src;
            src += 96;
        } else if (memcmp(y, leaf_value, 32) != 0) {
            return false;
        }
    }
    return true;
}

extern "C" int tc_verify_path_pairing(const tc_vkp* vkp, const tc_path* path, const uint8_t root[96],
                                      const uint8_t leaf_value[32], const void* proof, size_t proof_len) {
    try {
        if (!vkp || !path || !root || !leaf_value || !proof) return TC_ERR_ARG;
        PairingBatch B;
        if (!pairing_path_add(vkp, &B, *path, root, leaf_value, (const uint8_t*)proof, proof_len)) return TC_ERR_VERIFY;
        return pairing_batch_check(vkp, B) ? TC_OK : TC_ERR_VERIFY;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}

extern "C" int tc_verify_paths_pairing_batch(const tc_vkp* vkp, int count, const tc_path* paths, const uint8_t* roots,
                                             const uint8_t* leaf_values, const void* proofs, size_t proof_stride,
                                             const size_t* proof_len, int* results) {
    try {
        if (!vkp || count < 0 || (count && (!paths || !roots || !leaf_values || !proofs || !proof_len || !results))) return TC_ERR_ARG;
        if (!count) return TC_OK;
        /* the G1 work of the paths is spread over host threads, one running equation per thread */
        unsigned nthreads = std::min<unsigned>(std::max(1u, std::thread::hardware_concurrency()), 16u);
        nthreads = std::min<unsigned>(nthreads, (unsigned)count);
        std::vector<PairingBatch> part(nthreads);
        std::vector<uint8_t> structural(count, 0);
        auto work = [&](unsigned t) {
            for (int i = (int)t; i < count; i += (int)nthreads) {
                PairingBatch mine;                       /* a malformed path must not poison the thread's equation */
                bool ok = pairing_path_add(vkp, &mine, paths[i], roots + 96 * (size_t)i, leaf_values + 32 * (size_t)i,
                                           (const uint8_t*)proofs + (size_t)i * proof_stride, proof_len[i]);
                structural[i] = ok ? 1 : 0;
                if (!ok) continue;
                PairingBatch& P = part[t];
                bool unit = P.count == 0;
                uint32_t rho[4] = {1, 0, 0, 0};
                if (!unit)
                    for (int j = 0; j < 4; ++j) rho[j] = (uint32_t)P.rng();
                P.h_term = xyzz_add(P.h_term, weigh(mine.h_term, rho, unit));
                for (int j = 0; j < mine.m_used; ++j) P.tau_term[j] = xyzz_add(P.tau_term[j], weigh(mine.tau_term[j], rho, unit));
                P.m_used = std::max(P.m_used, mine.m_used);
                ++P.count;
            }
        };
        std::vector<std::thread> pool;
        for (unsigned t = 1; t < nthreads; ++t) pool.emplace_back(work, t);
        work(0);
        for (auto& th : pool) th.join();
        PairingBatch all;
        for (unsigned t = 0; t < nthreads; ++t) {
            if (!part[t].count) continue;
            bool unit = all.count == 0;
            uint32_t rho[4] = {1, 0, 0, 0};
            if (!unit)
                for (int j = 0; j < 4; ++j) rho[j] = (uint32_t)all.rng();
            all.h_term = xyzz_add(all.h_term, weigh(part[t].h_term, rho, unit));
            for (int j = 0; j < part[t].m_used; ++j) all.tau_term[j] = xyzz_add(all.tau_term[j], weigh(part[t].tau_term[j], rho, unit));
            all.m_used = std::max(all.m_used, part[t].m_used);
            ++all.count;
        }
        bool all_good = all.count == 0 || pairing_batch_check(vkp, all);
        for (int i = 0; i < count; ++i) {
            if (!structural[i]) { results[i] = TC_ERR_VERIFY; continue; }
            if (all_good) { results[i] = TC_OK; continue; }
            /* something in the batch is wrong: find out which paths, one by one */
            results[i] = tc_verify_path_pairing(vkp, paths + i, roots + 96 * (size_t)i, leaf_values + 32 * (size_t)i,
                                                (const uint8_t*)proofs + (size_t)i * proof_stride, proof_len[i]);
        }
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}

/* ======================================================================================= */
/* Layer selection: host only                                                              */
/* ======================================================================================= */
extern "C" int tc_hill_alpha(const double* eigenvalues, size_t d, size_t chi, double* out_alpha) {
    try {
        return selector::hill_alpha(eigenvalues, d, chi, out_alpha) ? TC_OK : TC_ERR_ARG;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}
extern "C" int tc_layer_benefits(const double* alpha, const double* params, size_t n_layers, double* out_nu) {
    try {
        if (!alpha || !params || !out_nu || !n_layers) return TC_ERR_ARG;
        selector::benefits(alpha, params, n_layers, out_nu);
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}
extern "C" int tc_select_layers(size_t n_layers, const double* nu, const double* phi, size_t n_verifiers, const double* beta,
                                double* out_value, int64_t* out_start, int64_t* out_end) {
    try {
        if (!nu || !phi || !beta || !out_value || !out_start || !out_end) return TC_ERR_ARG;
        if (n_layers > 0x7FFFFFFEull) return TC_ERR_SHAPE;
        for (size_t i = 0; i < n_layers; ++i)
            if (!(nu[i] >= 0.0) || !(phi[i] > 0.0)) return TC_ERR_RANGE;
        for (size_t k = 0; k < n_verifiers; ++k)
            if (!(beta[k] >= 0.0)) return TC_ERR_RANGE;
        *out_value = selector::select_layers(n_layers, nu, phi, n_verifiers, beta, out_start, out_end);
        return TC_OK;
    } catch (const std::bad_alloc&) {
        return TC_ERR_NOMEM;
    } catch (...) {
        return TC_ERR_STATE;
    }
}
