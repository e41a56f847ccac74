/*
 * tc.h -- C ABI of the MI355X tensor-commitment prover library (libtc.so).
 *
 * The library implements the prover-side hot path of TensorCommitments on one
 * gfx950 GPU: quantised tensor -> field elements -> tensor commitment (Def. 4.1,
 * Com) -> Terkle Tree of commitments (Sec. 4, Terkle Tree definition) ->
 * openings (Def. 4.1, Open; Terkle membership proof) -> path verification
 * (Def. 4.1, Ver in its sum form, checked with the trapdoor; Terkle verification).
 * Beyond that path, further down in this header: incremental updates of a tree, the
 * coefficient route of Def. 4.1 as printed (interpolation, Algorithm 1), and two parts
 * that run on the host only, as the paper's verifier has no GPU: verification with the
 * pairing and the layer selection of Sec. 4.3.
 *
 * Conventions
 *   - Every function returns TC_OK (0) or a negative TC_ERR_* code; nothing
 *     aborts or throws across this boundary.  tc_last_error(ctx) returns a
 *     human-readable message for the last failure on that context.
 *   - tc_ctx / tc_srs / tc_tree / tc_vk are opaque and owned by the library
 *     (create / destroy pairs).  All data buffers are owned by the caller.
 *   - Pointers named d_* are DEVICE pointers on the context's GPU; they are
 *     borrowed until the call returns (every call that returns bytes to the
 *     host synchronises the context's stream before returning).  All other
 *     pointers are HOST pointers.
 *   - Fr element: 32 bytes little-endian, value < r.  G1 element: 96 bytes
 *     x || y, 48 bytes little-endian each, affine, value < p; the point at
 *     infinity is 96 zero bytes.  Curve: BLS12-381 (App. E), commitments and
 *     proofs in G1.
 *   - Shapes are uint32_t[m], 1 <= m <= TC_MAX_ORDER, row-major with the last
 *     axis fastest (the lexicographic layout of App. A).  Grid positions are
 *     0-based; position i on an axis is the evaluation node zeta = i + 1.
 *   - One trapdoor vector (tau_1..tau_4) serves every shape of a context: axis
 *     j of any shape uses tau_j.
 *   - A context (its stream, workspace and staging memory) serves one host
 *     thread at a time; different contexts may be used from different threads
 *     at once, also on the same GPU and with shared tc_srs / tc_vk objects,
 *     which are read-only once built.  A tree belongs to the context that
 *     built it.  Kernels of contexts on different streams overlap only as far
 *     as the HIP runtime has hardware queues for them (GPU_MAX_HW_QUEUES, read
 *     when the runtime starts; its default is 4).
 */
#ifndef TC_H_
#define TC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TC_MAX_ORDER 4
#define TC_MAX_STEPS 16

#define TC_OK 0
#define TC_ERR_ARG (-1)    /* null pointer, bad enum, bad count */
#define TC_ERR_SHAPE (-2)  /* shape / order out of range or mismatching the SRS */
#define TC_ERR_RANGE (-3)  /* non-canonical field element, index outside the grid, trapdoor on the grid */
#define TC_ERR_NOMEM (-4)  /* host or device allocation failed */
#define TC_ERR_HIP (-5)    /* a HIP runtime call failed */
#define TC_ERR_VERIFY (-6) /* a proof was checked and rejected */
#define TC_ERR_STATE (-7)  /* object lacks what the call needs (e.g. SRS built without suffix tables) */

/* element types of caller buffers */
#define TC_I8 1  /* int8_t   */
#define TC_I16 2 /* int16_t  */
#define TC_FR 3  /* 32-byte canonical Fr elements */
#define TC_F16 4 /* IEEE binary16 (source type of tc_encode_tensor only) */

typedef struct tc_ctx tc_ctx;
typedef struct tc_srs tc_srs;
typedef struct tc_tree tc_tree;
typedef struct tc_vk tc_vk;

/* ---- context ----------------------------------------------------------------- */

/* Creates a context on GPU `device`.  `hip_stream` is a hipStream_t (as void*) on
 * which all work of this context is enqueued, or NULL for the default stream.
 * The stream stays owned by the caller.  Fails with TC_ERR_HIP when no GPU /
 * runtime is available: there is no CPU path. */
int tc_ctx_create(tc_ctx** out, int device, void* hip_stream);
void tc_ctx_destroy(tc_ctx* ctx);
const char* tc_last_error(const tc_ctx* ctx);
/* Blocks until all work enqueued by this context has finished. */
int tc_ctx_sync(tc_ctx* ctx);

/* Tuning options of a context.  The paper's own parameters are the security level, the shape and the arity
 * (Def. 4.1, Sec. 4); these are the knobs of this implementation of the multi-exponentiation.  0 = let the library
 * choose (the default for all of them).  At tc_ctx_create each option takes its value from the environment
 * variable named beside it when that is set to a valid number; tc_ctx_set_option overrides it afterwards.
 * A value outside the stated range is refused with TC_ERR_ARG and changes nothing.  Results do not depend on any
 * of them (the tests run the same commitments under several settings); tc_commit_static ignores them, its plan is
 * fixed by its scratch limit. */
#define TC_OPT_ACC_SUBRUN 0   /* TC_ACC_SUBRUN: entries per lane of the bucket accumulation, 1..64 */
#define TC_OPT_ACC_FANIN 1    /* TC_ACC_FANIN: partial sums per lane in the passes after it, 2..64 */
#define TC_OPT_FR_WINDOW 2    /* TC_FR_WINDOW: window width for full-width scalars, 8 or 16 bits */
#define TC_OPT_CHECK_LEVEL 3  /* TC_CHECK_LEVEL: 1 = every commitment that tc_commit / tc_commit_batch hand back is checked to
                                 lie on the curve (TC_ERR_STATE "internal" otherwise): a cheap guard while tuning */
#define TC_OPT_COUNT 4
int tc_ctx_set_option(tc_ctx* ctx, int option, int64_t value);
int tc_ctx_get_option(const tc_ctx* ctx, int option, int64_t* value);

/* Measurement hooks (for benchmarks; not part of the method).  With profiling enabled the
 * library brackets every launch of the selected kernel class with HIP events on the context's
 * stream; tc_ctx_profile_read synchronises, returns the summed duration and launch count since
 * the last read, and resets them. */
#define TC_PROF_BUCKET_ACC 0 /* bucket accumulation of tc_commit: one mixed addition per non-zero entry */
#define TC_PROF_NODE_COMMIT 1 /* bottom-level node commitments of an entries tree */
#define TC_PROF_NODE_COMMIT_UPPER 2 /* node commitments of the levels above (one launch per level) */
#define TC_PROF_VERIFY_CHAIN 3 /* doubling chains of path verification */
#define TC_PROF_KINDS 4
int tc_ctx_profile(tc_ctx* ctx, int enable);
int tc_ctx_profile_read(tc_ctx* ctx, int kind, double* total_ms, uint64_t* launches);
/* Work that the bracketed launches of a kind performed since the last call (then reset).  TC_PROF_BUCKET_ACC: the
 * mixed additions executed -- the non-zero terms minus the sub-runs they were cut into (the first term of a
 * sub-run is copied, and the sums of the sub-runs are added up by the passes that follow); 0 for the other kinds. */
int tc_ctx_profile_units(tc_ctx* ctx, int kind, uint64_t* units);

/* What the GPU's integer ALUs sustain, measured in place (the denominator of a roofline fraction for this path,
 * whose work is 32 x 32 + 64 -> 64 bit multiply-adds): a register-only loop with exactly `waves_per_simd` (1..8)
 * waves resident on every SIMD of the chip, timed with HIP events on the context's stream.
 *   TC_ALU_MAD        multiply-adds/s of independent v_mad_u64_u32 chains;
 *   TC_ALU_MAD_CARRY  the same with the carry of every multiply-add added into a third word, the pair of
 *                     instructions that a limb product of the field multiplication costs;
 *   TC_ALU_FP_MUL / TC_ALU_FP_SQR   Fp products / squarings per second of the library's own routines in a chain
 *                     (one product = 300 multiply-adds, one squaring 234);
 *   TC_ALU_FP_MUL_F64 / TC_ALU_FP_SQR_F64   the same for the exact variants on the FP64 pipe;
 *   TC_ALU_FP28_MUL / TC_ALU_FP28_SQR     the same for the carry-free form of the bucket accumulation (14 signed limbs
 *                     of 28 bits: 392 multiply-adds a product, 301 a squaring, no carry instructions). */
#define TC_ALU_MAD 0
#define TC_ALU_MAD_CARRY 1
#define TC_ALU_FP_MUL 2
#define TC_ALU_FP_SQR 3
#define TC_ALU_FP_MUL_F64 4
#define TC_ALU_FP_SQR_F64 5
#define TC_ALU_FP28_MUL 6
#define TC_ALU_FP28_SQR 7
int tc_ctx_alu_rate(tc_ctx* ctx, int kind, int waves_per_simd, double* out_per_s);

/* Test hook: one field operation per element on device arrays of raw limbs, little-endian 32-bit words, values
 * below the modulus (12 words per Fp element, 8 per Fr element), the Montgomery representatives that the kernels
 * keep in registers (radix R = 2^384 for Fp, 2^256 for Fr).  out[i] = op(a[i], b[i]), asynchronous on the context's
 * stream:  0 a b / R (the integer product routine)   1 a^2 / R   2, 3 the same through the FP64 pipe
 *          4 R^2 / a (inverse of a Montgomery representative, a != 0)   5 a b / R in Fr   6 a + b   7 a - b
 *          8 R^2 / a in Fr
 *          9 a b / R   10 a^2 / R   11 (a - b)(a + b) / R   12 (a - 2 b)(a - b) / R
 *          13 ((a - b)(a + b) - b (a - b)) / R: the 28-bit-limb form of the bucket accumulation (operands re-cut, sums
 *          and differences left unreduced with signed limbs, one product -- for 13 the difference of two products
 *          under one reduction --, back to the canonical element).
 * b is ignored by the one-operand operations but must be valid. */
int tc_ctx_field_op(tc_ctx* ctx, int op, const void* d_a, const void* d_b, size_t n, void* d_out);

/* ---- Setup (Def. 4.1, Setup) -- test-only trusted setup from a known trapdoor -- */

#define TC_SRS_SUFFIX 1u     /* also build the suffix tables S^(a), a = 1..m-1, needed by tc_open */
#define TC_SRS_FIXED_BASE 2u /* also build fixed-base window tables for every table (node shapes of a
                                tree: small shapes only, 50 MB per base) */
#define TC_SRS_OPEN_TABLE 8u /* also build the opening table of the leading axis, as large as the SRS itself,
                                U[kappa, t] = sum_(k != kappa) S[k, t] / (zeta_k - zeta_kappa),   t over the other axes:
                                a public linear image of the SRS.  With it an opening along the leading axis of a large
                                int8 / int16 tensor splits into the tensor's row commitments sum_t T[k, t] S[k, t], which
                                do not depend on the position (a tree keeps them per leaf tensor once computed), and one
                                short multi-exponentiation against row kappa of U.  The flag also keeps, behind the SRS
                                table, a copy of it multiplied by 2^8 (a second public image of the same size): the two
                                8-bit digits of an int16 entry then share one window of 128 buckets per row.  Shapes of
                                order >= 2 only; without it tc_open does the same work per opening.  Results are
                                identical either way. */
#define TC_SRS_MONOMIAL 4u   /* the monomial SRS of Def. 4.1 itself, S[k] = [prod_j tau_j^(k_j)] G, instead of its
                                Lagrange-basis image: for committing coefficient arrays (tc_interpolate,
                                tc_divide_by_linear) with tc_commit; not combinable with the other flags, and
                                tc_open / trees refuse it (TC_ERR_STATE) */

/* Builds, on the device, the Lagrange-basis SRS for `shape`:
 *   S[i] = [ prod_j l_{j,i_j}(tau_j) ] G,  i in prod_j {0..d_j-1},
 * the image of the monomial SRS of Def. 4.1 under the (public, linear) change of
 * basis; committing against it gives the same group element as interpolating and
 * committing against the monomial SRS.  tau: m canonical Fr values (m * 32 bytes);
 * a trapdoor that is 0 or lies on the grid {1..d_j} is rejected with TC_ERR_RANGE.
 * Device memory: 96 bytes per point of every table, and 128 more per point of S^(0) for the copy at a stride of
 * 128 bytes that the commitment kernels gather from (without memory for it they gather from the table itself). */
int tc_setup_from_trapdoor(tc_ctx* ctx, const uint8_t* tau, int m, const uint32_t* shape, uint32_t flags,
                           tc_srs** out);
void tc_srs_destroy(tc_srs* srs);
/* Number of points of table S^(first_axis) (prod of shape[first_axis..]); 0 if absent. */
uint64_t tc_srs_size(const tc_srs* srs, int first_axis);
/* Copies one SRS point to the host in canonical form (inspection / spot checks). */
int tc_srs_get_point(tc_ctx* ctx, const tc_srs* srs, int first_axis, uint64_t index, uint8_t out_g1[96]);

/* The public parameters as a flat file (Def. 4.1, Setup publishes pp = (srs, Omega): the SRS outlives the process
 * that made it).  Layout, little-endian: "TCSRS\0\0\0", u32 version (1), u32 curve (1 = BLS12-381 G1), u32 basis
 * (0 Lagrange image, 1 monomial), u32 flags, u32 m, u32 shape[4], u32 reserved, u64 point count; then the tables
 * S^(0) .. S^(m-1) that the SRS holds and, with TC_SRS_OPEN_TABLE, the opening table U, canonical 96-byte points.
 * Fixed-base tables, the grid constants and the 2^8-fold copy of S^(0) are not stored: the import rebuilds them.
 * Export: on entry *len is the capacity of host_buf, on return the size of the file; host_buf = NULL only asks for
 * the size; a buffer that is too small gives TC_ERR_ARG.
 * Import: builds an SRS equal to the exported one on this context's GPU.  A truncated or overlong buffer, a wrong
 * magic / version / curve, flags, shape or point count that do not fit together give TC_ERR_ARG or TC_ERR_SHAPE; a
 * point that is not canonical or not on the curve gives TC_ERR_RANGE.  (That the points are the powers of a
 * trapdoor nobody knows is the trusted party's promise; no check here can replace it.) */
int tc_srs_export(tc_ctx* ctx, const tc_srs* srs, void* host_buf, size_t* len);
int tc_srs_import(tc_ctx* ctx, const void* host_buf, size_t len, tc_srs** out);

/* ---- encode (quantisation + field embedding of the synthetic workloads) ------- */

/* d_src: n elements of `src_dtype`.  TC_F16: q = clamp(rint(float(x) * inv_scale), -32767, 32767)
 * (round half to even, one float32 multiply) written as int16 to d_dst.  TC_I8 / TC_I16: copied
 * unchanged to d_dst (same type).  The embedding e(q) = q mod r (negatives as r - |q|) is applied
 * inside the commitment kernels: -|q| P is computed as |q| (-P). */
int tc_encode_tensor(tc_ctx* ctx, const void* d_src, int src_dtype, size_t n, float inv_scale, void* d_dst);
/* The per-tensor scale of that rule, computed where the tensor is: d_inv_scale[0] (DEVICE memory, one float32,
 * 4-byte aligned) = float32(32767) / float32(amax), amax the largest magnitude among the finite values of the n
 * fp16 values at d_src; 0 when there is no non-zero finite value (every entry then quantises to 0).  Infinities and
 * NaNs do not count towards amax (they quantise to +-32767 and 0).  One pass over the tensor, asynchronous on the
 * context's stream; nothing is read back. */
int tc_quant_scale(tc_ctx* ctx, const void* d_src, size_t n, float* d_inv_scale);
/* tc_encode_tensor with the scale taken from device memory (what tc_quant_scale wrote, by launches that precede
 * this one on the stream): quantisation without a round trip to the host. */
int tc_encode_tensor_scaled(tc_ctx* ctx, const void* d_src, int src_dtype, size_t n, const float* d_inv_scale, void* d_dst);
/* tc_quant_scale followed by tc_encode_tensor_scaled (TC_F16) for `count` tensors in shared launches: the activations
 * of one forward pass are a hundred tensors of a few MB, and launched one by one their passes are bound by the
 * launches, not by HBM.  d_src[i]: n[i] fp16 values (device); d_inv_scale: `count` float32 in device memory, entry i
 * receives the scale of tensor i; d_dst[i]: n[i] int16 values (device).  The pointer arrays and n are host arrays.
 * Results are those of the two calls per tensor, bit for bit.  Asynchronous on the context's stream. */
int tc_encode_batch_scaled(tc_ctx* ctx, int count, const void* const* d_src, const size_t* n, float* d_inv_scale,
                           void* const* d_dst);

/* ---- Com (Def. 4.1, Com) -------------------------------------------------------- */

/* C_T = sum_i [e(T[i])] S[i] = g^{f_T(tau)}.  d_scalars: prod(shape) elements of `dtype`
 * (TC_I8, TC_I16 or TC_FR), laid out row-major.  Writes the canonical commitment. */
int tc_commit(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype, uint8_t out_g1[96]);
/* `count` independent commitments; out_g1 holds count * 96 bytes. */
int tc_commit_batch(tc_ctx* ctx, int count, const tc_srs* const* srs, const void* const* d_scalars,
                    const int* dtype, uint8_t* out_g1);

/* tc_commit for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The same commitment by the same kernels, but this call allocates nothing (no device memory,
 * no pinned memory, no events), reads nothing back and never waits for the stream: every intermediate lives in a
 * static device array of TC_STATIC_SCRATCH_BYTES that is part of the library (each GPU the library runs on holds
 * its copy until the process ends), and the canonical commitment is written to d_out_g1, a DEVICE buffer of 96
 * bytes (4-byte aligned) that is valid once the context's stream has reached this point.
 * Limits: dtype TC_I8 or TC_I16; at most TC_STATIC_MAX_TERMS entries (TC_ERR_SHAPE beyond that).
 * All contexts on one GPU share that GPU's array, which keeps the last call's contents: calls that overlap on one
 * GPU (different streams, different threads) race and must be serialised by the caller. */
#define TC_STATIC_MAX_TERMS (1u << 18)
#define TC_STATIC_SCRATCH_BYTES (32u << 20)
int tc_commit_static(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype, void* d_out_g1);
/* Number of allocations and releases of device or pinned host memory that the library has asked the HIP runtime
 * for since it was loaded (all contexts): a test hook for the promise above. */
uint64_t tc_alloc_calls(void);

/* ---- Open (Def. 4.1, Open; Algorithm 1 in evaluation form) ----------------------- */

/* Opens T at grid position kappa: y = T[kappa] and pi_i = g^{q_i(tau)}, i = 1..m, with
 * r_{i-1} = q_i (X_i - omega_i) + r_i.  The quotients are formed as values on the grid
 * (divided differences along axis i of the slice fixed by kappa_1..kappa_{i-1}) and
 * committed against the suffix table S^(i).  Needs TC_SRS_SUFFIX.  out_pi: m * 96 bytes. */
int tc_open(tc_ctx* ctx, const tc_srs* srs, const void* d_scalars, int dtype, const uint32_t* kappa,
            uint8_t out_y[32], uint8_t* out_pi);

/* ---- Ver (Def. 4.1, Ver, sum form; trapdoor-form check) --------------------------- */

/* Verification key of the test harness: the trapdoors themselves. */
int tc_vk_from_trapdoor(const uint8_t* tau, int m, tc_vk** out);
void tc_vk_destroy(tc_vk* vk);
/* Accepts (TC_OK) iff  C - [y]G == sum_i [tau_i - (kappa_i + 1)] pi_i  in G1, which holds iff
 * e(C g^{-y}, g) = prod_i e(pi_i, g^{tau_i - omega_i}).  Rejects with TC_ERR_VERIFY. */
int tc_verify(tc_ctx* ctx, const tc_vk* vk, int m, const uint32_t* shape, const uint8_t commitment[96],
              const uint32_t* kappa, const uint8_t y[32], const uint8_t* pi);

/* ---- Terkle Tree (Sec. 4: Terkle Tree, membership proof, verification) ------------- */

#define TC_LEAF_ENTRIES 0 /* bottom level = blocks of payload entries */
#define TC_LEAF_TENSORS 1 /* bottom level = whole tensors, one commitment each */

typedef struct tc_tree_desc {
    int m;                       /* order of the payload grid */
    uint32_t grid[TC_MAX_ORDER]; /* payload grid: entries (ENTRIES) or tensors (TENSORS) */
    uint32_t node_shape[TC_MAX_ORDER]; /* node shape d^(u) of every blocked level; arity B = prod */
    const tc_srs* node_srs;      /* SRS for node_shape, built with TC_SRS_SUFFIX | TC_SRS_FIXED_BASE */
    int leaf_kind;               /* TC_LEAF_ENTRIES or TC_LEAF_TENSORS */
    /* TC_LEAF_ENTRIES */
    const void* d_payload;       /* prod(grid) entries of `dtype` (TC_I8 / TC_I16), row-major */
    int dtype;
    /* TC_LEAF_TENSORS: prod(grid) tensors, row-major over the grid */
    const tc_srs* const* leaf_srs;      /* SRS of each tensor (its shape) */
    const void* const* d_leaf_scalars;  /* device buffer of each tensor */
    const int* leaf_dtype;
} tc_tree_desc;

/* Builds the tree level by level.  Level grids: ceil(grid / node_shape) per axis, repeated
 * until all ones; children outside the grid count as the field element 0; a child commitment
 * C enters its parent's tensor as phi(C) = (2 x_C + [y_C > (p-1)/2]) mod r, phi(O) = 0.
 * The payload / leaf buffers must stay valid for as long as openings are requested. */
int tc_terkle_build(tc_ctx* ctx, const tc_tree_desc* desc, tc_tree** out);
void tc_tree_destroy(tc_tree* tree);
int tc_terkle_root(const tc_tree* tree, uint8_t out_g1[96]);
/* Number of levels (bottom = 0, root level = levels - 1). */
int tc_terkle_levels(const tc_tree* tree);
/* Grid of a level (m entries) and its node count. */
int tc_terkle_level_info(const tc_tree* tree, int level, uint32_t* grid, uint64_t* n_nodes);
/* Commitment of node `index` (row-major in the level grid) in canonical form. */
int tc_terkle_node(tc_ctx* ctx, const tc_tree* tree, int level, uint64_t index, uint8_t out_g1[96]);

/* A built tree as a flat file, so that a later process can serve openings without rebuilding (Sec. 4: the tree is
 * built once per inference and opened on demand).  Layout, little-endian: "TCTREE\0\0", u32 version (1), u32 curve,
 * u32 m, u32 grid[4], u32 node_shape[4], u32 leaf kind, u32 levels, u32 reserved, u64 node count; then the canonical
 * 96-byte commitments of every node, level by level from the bottom, row-major in each level's grid.
 * Export: size protocol as tc_srs_export.
 * Import: `desc` describes the same tree as for tc_terkle_build (grid, node shape, node SRS, payload or leaf
 * tensors and their SRS on this GPU -- pointers and handles do not survive a process); the file must have been
 * written for that grid, node shape and leaf kind (TC_ERR_SHAPE otherwise; TC_ERR_ARG for a truncated, overlong or
 * foreign buffer; TC_ERR_RANGE for a point not on the curve).  The commitments are taken from the file, phi values
 * are recomputed; nothing checks that they are the commitments of the payload -- openings from a wrong file are
 * rejected by the verifier, as any wrong proof is. */
int tc_terkle_export(tc_ctx* ctx, const tc_tree* tree, void* host_buf, size_t* len);
int tc_terkle_import(tc_ctx* ctx, const tc_tree_desc* desc, const void* host_buf, size_t len, tc_tree** out);

/* Path of a payload position.  Steps run from the root down.  Step s opens a tensor of shape
 * shape[s] (order m[s]) at kappa[s]. */
typedef struct tc_path {
    int n_steps;
    int m[TC_MAX_STEPS];
    uint32_t shape[TC_MAX_STEPS][TC_MAX_ORDER];
    uint32_t kappa[TC_MAX_STEPS][TC_MAX_ORDER];
} tc_path;

/* Host-only: the path of `leaf_index` (m grid coordinates) in a tree over `grid` with uniform
 * `node_shape`.  For TC_LEAF_TENSORS the last step opens the leaf tensor (inner_m, inner_shape)
 * at inner_index; pass inner_m = 0 for TC_LEAF_ENTRIES. */
int tc_path_from_grid(int m, const uint32_t* grid, const uint32_t* node_shape, int leaf_kind,
                      const uint32_t* leaf_index, int inner_m, const uint32_t* inner_shape,
                      const uint32_t* inner_index, tc_path* out);

/* Membership proof.  Serialised top-down; step s contributes
 *     m[s] * 96 bytes  (pi_1..pi_m)  ||  32 bytes (opened value y)  ||  96 bytes (commitment of
 *     the next node on the path; absent in the last step).
 * On entry *proof_len is the capacity of proof_buf, on return the bytes written (TC_ERR_ARG with
 * the needed size in *proof_len if too small).  inner_index: position inside the leaf tensor
 * (TC_LEAF_TENSORS) or NULL. */
int tc_terkle_open(tc_ctx* ctx, const tc_tree* tree, const uint32_t* leaf_index, const uint32_t* inner_index,
                   void* proof_buf, size_t* proof_len);
/* `count` proofs at once; leaf_index / inner_index hold count * m (inner: count * inner order of
 * each leaf, concatenated); proofs are written at proof_buf + i * proof_stride, lengths to proof_len[i]. */
int tc_terkle_open_batch(tc_ctx* ctx, const tc_tree* tree, int count, const uint32_t* leaf_index,
                         const uint32_t* inner_index, void* proof_buf, size_t proof_stride, size_t* proof_len);

/* Walks the path from the root: every opening must verify against the commitment carried down,
 * every opened value above the bottom must equal phi(next commitment), the bottom value must equal
 * leaf_value, and the chain must start at `root`.  TC_OK = accept, TC_ERR_VERIFY = reject. */
int tc_verify_path(tc_ctx* ctx, const tc_vk* vk, const tc_path* path, const uint8_t root[96],
                   const uint8_t leaf_value[32], const void* proof, size_t proof_len);
/* `count` paths on the GPU at once; results[i] = TC_OK or TC_ERR_VERIFY.  Returns TC_OK when the
 * batch ran (whatever the verdicts). */
int tc_verify_paths_batch(tc_ctx* ctx, const tc_vk* vk, int count, const tc_path* paths, const uint8_t* roots,
                          const uint8_t* leaf_values, const void* proofs, size_t proof_stride,
                          const size_t* proof_len, int* results);

/* One entry changed by `delta` (new value minus old value): recomputes the commitments on its path only,
 * reusing the rest of the tree (Sec. 4.2): C' = C + [delta] S[k] for the node (entries tree) or the leaf tensor
 * (tensors tree: inner_index is the entry's position in that tensor, else NULL) that holds the entry, then
 * C' = C + [phi(child') - phi(child)] S[k] level by level up to the root.  The caller writes the new value into
 * its own payload / tensor buffer (before or after this call; openings read that buffer).  |delta| < 2^32.
 * Blocked levels need the fixed-base node SRS (TC_ERR_STATE otherwise). */
int tc_terkle_update(tc_ctx* ctx, tc_tree* tree, const uint32_t* leaf_index, const uint32_t* inner_index, int64_t delta);

/* ---- the coefficient route: interpolation and Algorithm 1 on the device -----------------------
 *
 * Def. 4.1 commits to the monomial coefficients of the interpolant f_T; the hot path above never forms them
 * (a Lagrange-basis SRS gives the same group element).  These two calls are the literal route.  Coefficient
 * arrays have the tensor's shape, row-major (entry k = coefficient of prod_j x_j^(k_j)), canonical Fr values of
 * 32 bytes, device memory. */

/* d_coeffs = monomial coefficients of the polynomial with f(zeta) = T[zeta] on the grid prod_j {1..d_j}
 * (Sec. 4, Com; one axis at a time in Newton form, App. C: divided differences on the equispaced nodes, then
 * expansion of the nested products).  m <= TC_MAX_INTERP_ORDER axes; the scalars as in tc_commit. */
#define TC_MAX_INTERP_ORDER 12
int tc_interpolate(tc_ctx* ctx, int m, const uint32_t* shape, const void* d_scalars, int dtype, void* d_coeffs);
/* The same coefficients through one of the three interpolation forms of App. C, the comparison of Fig. 1:
 * Newton (divided differences; what tc_interpolate uses), Gregory (forward differences Delta^k T[0] on the
 * equispaced grid, weights binom(X - zeta_0, k)) or barycentric (weights beta_l, the interpolant assembled as
 * sum_l beta_l T_l prod_(r != l) (X - zeta_r) node by node).  All three return the identical array; they differ
 * in their steps and running time.  The barycentric form needs five Fr arrays of the tensor's size as
 * workspace, the others three.  Unknown form: TC_ERR_ARG. */
#define TC_INTERP_NEWTON 0
#define TC_INTERP_GREGORY 1
#define TC_INTERP_BARYCENTRIC 2
int tc_interpolate_form(tc_ctx* ctx, int m, const uint32_t* shape, const void* d_scalars, int dtype, int form,
                        void* d_coeffs);
/* Algorithm 1 (App. A): f = q (x_axis - omega) + r with omega = kappa_axis + 1 and r free of x_axis, on the
 * coefficient arrays; d_quotient and d_remainder have the full shape (zeros at the top degree of the axis in q,
 * at every positive degree in r) and may not alias d_coeffs. */
int tc_divide_by_linear(tc_ctx* ctx, int m, const uint32_t* shape, const void* d_coeffs, int axis, uint32_t kappa_axis,
                        void* d_quotient, void* d_remainder);

/* ---- public verification with the pairing (CPU only) ----------------------------------------
 *
 * The pairing form of Ver (Def. 4.1; the bilinear map of App. E) in the sum form used throughout:
 *     e(C - [y]G, H) = prod_i e(pi_i, [tau_i]H - [zeta_i]H),   zeta_i = kappa_i + 1,
 * with H the generator of G2 and [tau_i]H part of the public parameters: no trapdoor is needed to verify.
 * The paper's verifier has no GPU; these calls run on the host, need no context and never touch the HIP
 * runtime.  G2 points: 192 bytes = x.c0, x.c1, y.c0, y.c1 (x = x.c0 + x.c1 u), canonical, 48 bytes
 * little-endian each, all zero for the identity.  Target-group elements: 576 bytes = the twelve Fp coefficients of
 * w^0 .. w^11 in Fp[w]/(w^12 - 2 w^6 + 2), 48 bytes little-endian each.  Points must lie on their curves
 * (checked); membership in the prime-order subgroups is not checked. */
typedef struct tc_vkp tc_vkp;

/* Test-only setup of the public verification key [tau_i]H, i < m <= TC_MAX_ORDER, from the trapdoor
 * (m canonical 32-byte Fr values).  TC_ERR_ARG / TC_ERR_RANGE / TC_ERR_NOMEM. */
int tc_vkp_from_trapdoor(const uint8_t* tau, int m, tc_vkp** out);
void tc_vkp_destroy(tc_vkp* vkp);
/* out_g2 = [tau_axis]H, or H for axis = -1 */
int tc_vkp_get(const tc_vkp* vkp, int axis, uint8_t out_g2[192]);
/* out_gt = e(P, Q) = f_{|z|,Q}(P)^(-(p^12 - 1)/r) (z < 0 the curve parameter); the identity on either side gives 1.
 * TC_ERR_ARG for a null pointer, TC_ERR_RANGE for a point that is not canonical or not on its curve. */
int tc_pairing(const uint8_t p_g1[96], const uint8_t q_g2[192], uint8_t out_gt[576]);
/* Ver for one opening; arguments as tc_verify.  TC_OK, TC_ERR_VERIFY (including malformed points), or
 * TC_ERR_ARG / TC_ERR_SHAPE / TC_ERR_RANGE for bad arguments. */
int tc_verify_pairing(const tc_vkp* vkp, int m, const uint32_t* shape, const uint8_t commitment[96],
                      const uint32_t* kappa, const uint8_t y[32], const uint8_t* pi);
/* Path verification as tc_verify_path, with the pairing and phi on the host.  The equations of the steps are
 * combined with random 128-bit weights into one check (m + 1 Miller loops and one final exponentiation for the
 * whole path): a path with a wrong step is accepted with probability about 2^-128. */
int tc_verify_path_pairing(const tc_vkp* vkp, const tc_path* path, const uint8_t root[96],
                           const uint8_t leaf_value[32], const void* proof, size_t proof_len);

/* Many paths at once, arguments as tc_verify_paths_batch: the equations of all well-formed paths are combined
 * (random weights again) into one check, their G1 arithmetic spread over up to 16 host threads; only when that
 * check fails are the paths verified one by one to find the wrong ones.  results[i] = TC_OK or TC_ERR_VERIFY. */
int tc_verify_paths_pairing_batch(const tc_vkp* vkp, int count, const tc_path* paths, const uint8_t* roots,
                                  const uint8_t* leaf_values, const void* proofs, size_t proof_stride,
                                  const size_t* proof_len, int* results);

/* ---- layer selection (CPU only; the verifier's policy, Sec. 4.3) --------------------------------
 * float64; no context, no GPU. */

/* Hill estimator of the tail exponent on the chi largest of d eigenvalues (any order):
 * alpha = 1 + chi / sum_{r=1..chi} ln(Lambda_{d-r+1} / Lambda_{d-chi}).  TC_ERR_ARG unless 1 <= chi < d and the
 * eigenvalue Lambda_{d-chi} is positive and the tail is not flat. */
int tc_hill_alpha(const double* eigenvalues, size_t d, size_t chi, double* out_alpha);
/* nu_i = (alpha_max - alpha_i) / (alpha_max - alpha_min) * P_i / sum_j P_j (all zero when every alpha is equal) */
int tc_layer_benefits(const double* alpha, const double* params, size_t n_layers, double* out_nu);
/* Problem 4.5 by the dynamic program of App. D in O(M L) time: verifier k (budget beta[k]) takes no layers or one
 * contiguous interval [out_start[k], out_end[k]] (0-based, inclusive; -1, -1 for none) of cost at most beta[k],
 * intervals disjoint and in the order of the verifiers; out_value = total benefit.  The recursion also lets a
 * verifier stay idle (DP[k-1, i]), which the printed one omits.  nu >= 0, phi > 0, beta >= 0 (TC_ERR_RANGE). */
int tc_select_layers(size_t n_layers, const double* nu, const double* phi, size_t n_verifiers, const double* beta,
                     double* out_value, int64_t* out_start, int64_t* out_end);

#ifdef __cplusplus
}
#endif
#endif /* TC_H_ */
