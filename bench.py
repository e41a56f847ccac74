#!/usr/bin/env python3
"""Benchmark of the TensorCommitments prover hot path on one MI355X.

A step is one pass of the whole path over one synthetic LLaMA2-7B-shaped forward
(32 layers x {512x4096, 512x4096, 512x11008} fp16 N(0,1) activations, 314 572 800
entries): per-tensor scale and quantisation on the GPU, one tensor commitment per
tensor, the arity-16 Terkle tree over the 96 commitments, the configuration's 64
random path openings down to tensor entries, and their batch verification.  All
inputs and the SRS tables are resident in HBM before the timed region.

Prints one JSON line: metric "tensor elements committed/sec" over the whole step,
`terkle_build_ms_per_llama2_7b_fwd` (scale + quantisation + tree build, the second
half of the metric), `roofline` (integer-ALU bound, the bucket-accumulation launch
of the build, against the multiply-add rate measured in the same run: `alu_peak`),
and `cpu_baseline` (the CPU oracle's naive multi-exponentiation on bounded samples
of the single-layer tensor).  The single-layer step of the previous headline is
kept as the sub-object `c2_step`.
"""
import argparse
import ctypes
import json
import os
import sys
import time

# Steps in flight (the c2_step leg) run on streams of their own, and streams that share a hardware queue run
# their kernels one after the other.  HIP's default of 4 queues per process caps the overlap of that leg's many
# short, latency-bound kernels (2.69 ms per step with 4 queues and 4 steps in flight, 2.03 ms with 16 and 12).
# The runtime reads the variable when it starts, so it is set before anything loads HIP (TC_BENCH_HW_QUEUES
# overrides the count).
os.environ["GPU_MAX_HW_QUEUES"] = os.environ.get("TC_BENCH_HW_QUEUES", "16")

import numpy as np  # noqa: E402

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import tc_inputs  # noqa: E402

# One mixed addition in XYZZ coordinates = 8 multiplications + 2 squarings in Fp; one
# Montgomery product of 12 x 32-bit limbs = 2 * 12^2 + 12 = 300 32x32->64 multiply-adds.
FP_MULS_PER_MIXED_ADD = 10
MADS_PER_FP_MUL = 300
# What the accumulation kernel issues per mixed addition: it computes in 14 limbs of 28 bits (no carry
# instructions), 392 multiply-adds a product, 301 a squaring, 588 for the difference of two products under one
# reduction: 6 products + 2 squarings + 1 such difference.
MADS_ISSUED_PER_MIXED_ADD = 6 * 392 + 2 * 301 + 588
# Integer-ALU peak by the formula: v_mad_u64_u32 at half the full vector rate, 256 CU x 4 SIMD x 16 lanes x
# 2.4 GHz / 2.  Printed beside the rate that `alu_peak` measures in the same run, which is the denominator used.
FORMULA_PEAK_MADS_PER_S = 256 * 4 * 16 * 2.4e9 / 2
R_MODULUS = 0x73EDA753299D7D483339D80809A1D80553BDA402FFFE5BFEFFFFFFFF00000001      # group order (embedding of negatives)
# HBM bytes moved by the bucket-accumulation launch of one LLaMA2-7B-shaped build (rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE of `bench.py --only-c3-build`, scaled by a 256 MiB copy kernel; runs and scale factors in
# profiles/c3_build_hbm_traffic_pmc.txt).
ACC_TRAFFIC_BYTES_C3 = 5.179e10
# Vector instructions that the same launch issues per SIMD and clock, and per mixed addition (rocprofv3 --pmc
# SQ_INSTS_VALU / GRBM_GUI_ACTIVE of the same command: profiles/c3_build_sq_counters_pmc.txt).  A 64-lane wave takes
# four clocks of a 16-lane SIMD, so 0.25 is the most a SIMD can issue.
ACC_VALU_PER_SIMD_CLK_C3 = 0.245
ACC_VALU_PER_ADDITION_C3 = 4777


# ----------------------------------------------------------------------------------------------------------
# measured integer-ALU peak
# ----------------------------------------------------------------------------------------------------------
def alu_peak(ctx, T):
    """Multiply-add rates of register-only loops on every SIMD of the chip, at 1 / 2 / 4 / 8 waves per SIMD: pure
    v_mad_u64_u32 chains, the multiply-add + carry-add pair of a limb product, and the library's own Fp product
    and squaring in a chain (x 300 and x 234 multiply-adds).  `used` is the best pure rate: the roofline's peak."""
    B = T.binding
    out = {"unit": "32x32+64 multiply-adds/s", "formula": FORMULA_PEAK_MADS_PER_S,
           "formula_note": "256 CU x 4 SIMD x 16 lanes x 2.4 GHz / 2 (v_mad_u64_u32 at half rate)",
           "mad_u64_u32": {}, "mad_plus_carry_add": {}, "fp_mul_products_per_s": {}, "fp_sqr_squarings_per_s": {},
           "fp_mul_f64_products_per_s": {}, "fp_sqr_f64_squarings_per_s": {},
           "fp28_mul_products_per_s": {}, "fp28_sqr_squarings_per_s": {}}
    for w in (1, 2, 4, 8):
        out["mad_u64_u32"][str(w)] = ctx.alu_rate(B.TC_ALU_MAD, w)
        out["mad_plus_carry_add"][str(w)] = ctx.alu_rate(B.TC_ALU_MAD_CARRY, w)
    for w in (1, 2, 3, 4):
        out["fp_mul_products_per_s"][str(w)] = ctx.alu_rate(B.TC_ALU_FP_MUL, w)
        out["fp_sqr_squarings_per_s"][str(w)] = ctx.alu_rate(B.TC_ALU_FP_SQR, w)
        out["fp28_mul_products_per_s"][str(w)] = ctx.alu_rate(B.TC_ALU_FP28_MUL, w)
        out["fp28_sqr_squarings_per_s"][str(w)] = ctx.alu_rate(B.TC_ALU_FP28_SQR, w)
    for w in (1, 2):                                   # the FP64-pipe variants serve depth-bound chains of few waves
        out["fp_mul_f64_products_per_s"][str(w)] = ctx.alu_rate(B.TC_ALU_FP_MUL_F64, w)
        out["fp_sqr_f64_squarings_per_s"][str(w)] = ctx.alu_rate(B.TC_ALU_FP_SQR_F64, w)
    out["used"] = max(out["mad_u64_u32"].values())
    best_mul = max(out["fp_mul_products_per_s"].values())
    out["fp_mul_frac_of_used"] = best_mul * MADS_PER_FP_MUL / out["used"]
    out["note"] = ("keys = waves per SIMD; `used` (best pure multiply-add rate) is the denominator of every "
                   "roofline fraction of this line; fp_mul_frac_of_used = what the product routine reaches of it in isolation")
    return out


# ----------------------------------------------------------------------------------------------------------
# headline: the LLaMA2-7B-shaped forward
# ----------------------------------------------------------------------------------------------------------
class C3Forward:
    """Inputs, SRS tables and buffers of the LLaMA2-7B-shaped forward, resident on the device."""

    def __init__(self, ctx, T, torch, node_srs, tau):
        self.ctx, self.T, self.torch, self.node_srs = ctx, T, torch, node_srs
        cfg = tc_inputs.LLAMA7B
        self.shapes3 = tc_inputs.c3_shapes(cfg)
        self.srs_by_shape = {s: ctx.setup_from_trapdoor(tau, s, T.TC_SRS_SUFFIX | T.TC_SRS_OPEN_TABLE) for s in set(self.shapes3)}
        gen = torch.Generator(device="cuda")
        gen.manual_seed(tc_inputs.tensor_seed(2))
        self.xs, self.qs, self.leaf_srs = [], [], []
        for _layer in range(cfg["layers"]):
            for s in self.shapes3:
                x = torch.randn(s[0] * s[1], generator=gen, device="cuda", dtype=torch.float32).to(torch.float16)
                self.xs.append(x)
                self.qs.append(torch.empty(x.numel(), dtype=torch.int16, device="cuda"))
                self.leaf_srs.append(self.srs_by_shape[s])
        self.scales = torch.zeros(len(self.xs), dtype=torch.float32, device="cuda")
        self.total = sum(x.numel() for x in self.xs)
        self.grid = (cfg["layers"], 3)
        rng = np.random.default_rng(tc_inputs.tensor_seed(2) + 999)
        self.leaves = [(int(rng.integers(0, self.grid[0])), int(rng.integers(0, 3))) for _ in range(64)]
        self.inners = [tuple(int(rng.integers(0, d)) for d in self.shapes3[l[1]]) for l in self.leaves]
        self.vk = ctx.vk_from_trapdoor(tau)
        self.dtypes = [T.TC_I16] * len(self.qs)
        torch.cuda.synchronize()

    def quantise(self):
        """A1 / A2: per-tensor scale (one pass) and quantisation (one pass), all on the device"""
        self.ctx.encode_batch_scaled(self.xs, [x.numel() for x in self.xs], self.scales, self.qs)

    def build(self):
        """A4 - A6: 96 leaf commitments and the upper levels; returns when the root is on the host"""
        return self.ctx.terkle_build_tensors(self.node_srs, self.leaf_srs, self.qs, self.dtypes, self.grid, tc_inputs.NODE_SHAPE)

    def leaf_values(self):
        torch = self.torch
        flat = torch.stack([self.qs[l[0] * 3 + l[1]][i[0] * self.shapes3[l[1]][1] + i[1]] for l, i in zip(self.leaves, self.inners)])
        return [(int(v) % R_MODULUS).to_bytes(32, "little") for v in flat.cpu().tolist()]

    def step(self, times=None):
        """One pass of the whole path.  `times`, when given, collects host-clock marks at the phase boundaries
        (each of build / open / verify returns only when its result bytes are on the host)."""
        t0 = time.perf_counter()
        self.quantise()
        tree = self.build()
        t1 = time.perf_counter()
        proofs = tree.open_batch(self.leaves, self.inners)
        t2 = time.perf_counter()
        if self.paths is None:
            self.paths = [tree.path(l, i) for l, i in zip(self.leaves, self.inners)]
        root = tree.root
        ok = self.ctx.verify_paths_batch(self.vk, self.paths, [root] * 64, self.values, proofs)
        t3 = time.perf_counter()
        tree.close()
        if times is not None:
            times.append((t1 - t0, t2 - t1, t3 - t2))
        return root, ok

    paths = None
    values = None

    def close(self):
        for s in self.srs_by_shape.values():
            s.close()


def bench_c3(ctx, T, torch, node_srs, tau, steps, warmup, peak):
    B = T.binding
    fwd = C3Forward(ctx, T, torch, node_srs, tau)
    fwd.quantise()
    ctx.sync()
    fwd.values = fwd.leaf_values()
    for _ in range(max(warmup, 1)):
        root0, ok = fwd.step()
        assert all(ok), "C3 openings failed verification"
    torch.cuda.synchronize()
    # timed region: exactly `steps` passes of the whole path, wall clock between two device synchronisations
    marks = []
    t0 = time.perf_counter()
    for _ in range(steps):
        root, ok = fwd.step(marks)
        assert root == root0 and all(ok)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    build_ms = sorted(m[0] for m in marks)[len(marks) // 2] * 1e3
    open_ms = sorted(m[1] for m in marks)[len(marks) // 2] * 1e3
    verify_ms = sorted(m[2] for m in marks)[len(marks) // 2] * 1e3
    # the quantisation passes alone (HBM-bound: 2 B read for the scale; 2 B read + 2 B written for the values)
    torch.cuda.synchronize()
    tq = time.perf_counter()
    for _ in range(3):
        fwd.quantise()
    ctx.sync()
    quant_ms = (time.perf_counter() - tq) * 1e3 / 3
    # a second, untimed pass with HIP events around the bucket-accumulation launch of the build
    ctx.profile_read(B.TC_PROF_BUCKET_ACC)
    ctx.profile_units(B.TC_PROF_BUCKET_ACC)
    ctx.profile(True)
    prof_builds = 3
    for _ in range(prof_builds):
        fwd.quantise()
        fwd.build().close()
    acc_ms, acc_launches = ctx.profile_read(B.TC_PROF_BUCKET_ACC)
    acc_executed = ctx.profile_units(B.TC_PROF_BUCKET_ACC) / max(acc_launches, 1)
    ctx.profile(False)
    nonzero = sum(int(torch.count_nonzero(q).item()) for q in fwd.qs)
    kern_ms = acc_ms / max(acc_launches, 1)
    per_add = FP_MULS_PER_MIXED_ADD * MADS_PER_FP_MUL
    achieved = acc_executed * per_add / (kern_ms * 1e-3)
    # public verification of the same 64 paths with the pairing, on the host (the paper's verifier has no GPU)
    tree = fwd.build()
    proofs = tree.open_batch(fwd.leaves, fwd.inners)
    pv = B.PairingVerifier(tau, 2)
    t5 = time.perf_counter()
    ok_pv = pv.verify_paths(fwd.paths, [tree.root] * 64, fwd.values, proofs)
    public_ms = (time.perf_counter() - t5) * 1e3
    pv.close()
    tree.close()
    assert all(ok_pv), "C3 openings failed public verification"
    out = {
        "value": fwd.total * steps / elapsed,
        "ms_per_step": elapsed * 1e3 / steps,
        "elements": fwd.total,
        "terkle_build_ms_per_llama2_7b_fwd": build_ms,
        "build_elements_per_s": fwd.total / (build_ms * 1e-3),
        "phase_ms": {"scale+quantise+build": build_ms, "open_64_paths": open_ms, "verify_64_paths": verify_ms,
                     "scale+quantise_alone": quant_ms},
        "quantise_stream": {"bound": "hbm", "bytes": 6.0 * fwd.total, "ms": quant_ms, "achieved": 6.0 * fwd.total / (quant_ms * 1e-3) / 1e9,
                            "peak": 8000.0, "unit": "GB/s", "frac": 6.0 * fwd.total / (quant_ms * 1e-3) / 8e12,
                            "note": "tc_encode_batch_scaled: the scales (2 B read per element), then the values (2 B read, 2 B written), 96 tensors in shared launches"},
        "public_verify_64_paths_host_ms": public_ms,
        "roofline": {"bound": "alu", "achieved": achieved / 1e12, "peak": peak / 1e12, "unit": "T 32x32->64 multiply-add/s",
                     "frac": achieved / peak, "traffic": ACC_TRAFFIC_BYTES_C3,
                     "traffic_unit": "HBM bytes per launch (fetch + write)",
                     "kernel": "AccAffine (bucket accumulation of all 96 leaf commitments, one launch per build)",
                     "kernel_ms": kern_ms, "launches": acc_launches,
                     # `achieved` counts the mixed additions that the launch itself executes (the first entry of a
                     # sub-run is a copy; the passes after it add the sub-run sums up), 3000 multiply-adds each
                     "mixed_additions_executed_per_launch": acc_executed,
                     "nonzero_entries_per_launch": nonzero,
                     "peak_source": "alu_peak.used, measured in this run",
                     "frac_of_formula_peak": achieved / FORMULA_PEAK_MADS_PER_S,
                     # the unit of `achieved` is the algorithm's count (10 Fp products x 300 multiply-adds at 32-bit
                     # limbs); the kernel's own 28-bit-limb products issue more multiply-adds for the same addition
                     "multiply_adds_issued_per_addition": MADS_ISSUED_PER_MIXED_ADD,
                     "issue_frac": acc_executed * MADS_ISSUED_PER_MIXED_ADD / (kern_ms * 1e-3) / peak,
                     "issue_frac_note": "multiply-adds the launch really issues over the measured multiply-add peak",
                     "valu_issue": {"per_simd_clk": ACC_VALU_PER_SIMD_CLK_C3, "max": 0.25,
                                    "vector_instructions_per_addition": ACC_VALU_PER_ADDITION_C3,
                                    "source": "profiles/c3_build_sq_counters_pmc.txt",
                                    "note": "the launch issues a vector instruction on every SIMD every four clocks: "
                                            "only fewer instructions per addition can make it faster"},
                     "build_frac": nonzero * per_add / (build_ms * 1e-3) / peak,
                     "build_frac_note": "one mixed addition per non-zero entry over the whole scale + quantise + build time"},
    }
    fwd.close()
    return out


def only_c3_build(ctx, T, torch, node_srs, tau, builds):
    """Profiling mode: nothing but set-up and `builds` quantise + build passes of the LLaMA2-7B-shaped forward, so
    that a rocprofv3 kernel trace of the run holds only those launches."""
    fwd = C3Forward(ctx, T, torch, node_srs, tau)
    roots = []
    for _ in range(builds):
        fwd.quantise()
        tree = fwd.build()
        roots.append(tree.root)
        tree.close()
    ctx.sync()
    assert len(set(roots)) == 1
    fwd.close()
    print(json.dumps({"mode": "only-c3-build", "builds": builds, "elements": fwd.total}))


# ----------------------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands
# ----------------------------------------------------------------------------------------------------------
def cpu_baseline(q):
    """The oracle's naive multi-exponentiation (every term its own double-and-add over the Lagrange SRS, route (b))
    on the first 2^12 and 2^14 entries of the quantised single-layer tensor, on one core and on all the cores the
    box gives us; linear extrapolation to the configurations, labelled as such; the trapdoor closed form (route
    (c), not an MSM: it uses the trapdoor) timed on the whole tensor beside it."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import bls12_381 as ec
    from oracle import cbind, tc

    cores = min(os.cpu_count() or 1, 16)
    shape = tc_inputs.C2_SHAPE
    pp = tc.setup(shape, tc_inputs.trapdoors())
    flat = q.reshape(-1)
    n_big, n_small = 1 << 14, 1 << 12
    cbind.lib()
    t0 = time.time()
    with ThreadPoolExecutor(max_workers=cores) as pool:       # SRS points of the sample by the oracle's own scalar multiplication
        pts = b"".join(pool.map(lambda f: ec.g1_to_bytes(cbind.g1_mul(pp.lagrange_scalar(tc.multi_index(f, shape)), ec.G1)), range(n_big)))
    srs_s = time.time() - t0
    runs = {}
    used_all = cores
    for n in (n_small, n_big):
        sample = np.ascontiguousarray(flat[:n])
        for threads in (1, cores):
            # bounded: one pass on one core; on all cores passes are repeated for about three seconds of wall clock
            # (about ten seconds for the whole baseline, its sample SRS included)
            t0, reps = time.time(), 0
            while True:
                _, used = cbind.msm_naive(sample, pts[: 96 * n], threads)
                reps += 1
                dt = time.time() - t0
                if threads == 1 or dt > 3.0:
                    break
            runs["%d_entries_%s" % (n, "1_core" if threads == 1 else "all_cores")] = {
                "seconds": dt, "passes": reps, "scalars_per_s": n * reps / dt, "threads": used}
            if threads != 1:
                used_all = used
    t0 = time.time()
    cbind.commit(pp, q, cores)
    route_c_s = time.time() - t0
    best = runs["%d_entries_all_cores" % n_big]["scalars_per_s"]
    one = runs["%d_entries_1_core" % n_big]["scalars_per_s"]
    sizes = {"C2": 2097152, "C3": 314572800, "C4": 6476005376, "C5": 15770583040}
    return {
        "value": best,
        "unit": "tensor elements committed/sec",
        "cores": used_all,
        "kind": "oracle",
        "sample": "naive double-and-add multi-exponentiation (commitment only, no tree) over the first 2^14 entries of the "
                  "quantised 512x4096 int16 tensor, %d threads; also 2^12 entries and one core in `runs`" % used_all,
        "one_core_scalars_per_s": one,
        "runs": runs,
        "sample_srs_seconds": srs_s,
        "extrapolated_seconds_all_cores": {k: v / best for k, v in sizes.items()},
        "extrapolated_seconds_one_core": {k: v / one for k, v in sizes.items()},
        "extrapolation_note": "linear in the entry count from the 2^14-entry sample: an extrapolation, not a measurement",
        "trapdoor_closed_form_c2_seconds": route_c_s,
        "trapdoor_closed_form_note": "route (c): field sums + one scalar multiplication, all cores; uses the trapdoor, so it "
                                     "is the parity route and not an MSM baseline",
    }


# ----------------------------------------------------------------------------------------------------------
# sub-objects: the single-layer step with steps in flight, and the widened rows
# ----------------------------------------------------------------------------------------------------------
def hip_event_timer():
    """HIP events through the runtime library directly (the library's stream is the default stream)."""
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    return hip


class Events:
    def __init__(self, hip):
        self.hip = hip
        self.pairs = []

    def start(self):
        a, b = ctypes.c_void_p(), ctypes.c_void_p()
        self.hip.hipEventCreate(ctypes.byref(a))
        self.hip.hipEventCreate(ctypes.byref(b))
        self.hip.hipEventRecord(a, None)
        return (a, b)

    def stop(self, pair):
        self.hip.hipEventRecord(pair[1], None)
        self.pairs.append(pair)

    def total_ms(self):
        tot = 0.0
        for a, b in self.pairs:
            self.hip.hipEventSynchronize(b)
            ms = ctypes.c_float()
            self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
            tot += ms.value
        return tot


def bench_c2_step(ctx, T, torch, lib, node_srs, tau, steps, warmup, in_flight, openings, peak):
    """The single-layer configuration: quantise a 512 x 4096 activation, commit it as one tensor commitment
    (second stream), build the (4,4) tree over its 2^21 entries, open `openings` paths and verify them, with
    `in_flight` such steps in flight on streams of their own.  Returns the sub-object and the quantised tensor."""
    import queue
    import threading

    B = T.binding
    shape, node = tc_inputs.C2_SHAPE, tc_inputs.NODE_SHAPE
    n = shape[0] * shape[1]
    srs = ctx.setup_from_trapdoor(tau, shape, 0)
    x = tc_inputs.c2_activation()
    dx = torch.from_numpy(x.view(np.int16)).cuda()
    leaves = tc_inputs.opening_positions(shape, openings, tc_inputs.tensor_seed(1))
    vk = ctx.vk_from_trapdoor(tau)
    paths = [ctx.path_from_grid(shape, node, T.TC_LEAF_ENTRIES, l) for l in leaves]
    torch.cuda.synchronize()

    class Lane:
        """One step in flight: a main context (tree, openings, verification) and a side context on its own
        default-priority stream for the flat commitment, which a long-lived host thread drives."""

        def __init__(self, main_ctx):
            self.own_ctx = main_ctx is None
            if main_ctx is None:
                self.main_stream = torch.cuda.Stream()
                main_ctx = T.Context(0, self.main_stream.cuda_stream, lib)
            self.ctx = main_ctx
            self.side_stream = torch.cuda.Stream()
            self.ctx2 = T.Context(0, self.side_stream.cuda_stream, lib)
            self.dq = torch.empty(n, dtype=torch.int16, device="cuda")
            self.scale = torch.zeros(1, dtype=torch.float32, device="cuda")
            self.jobs, self.done = queue.Queue(), queue.Queue()
            self.thread = threading.Thread(target=self.side_worker, daemon=True)
            self.thread.start()

        def side_worker(self):
            while True:
                job = self.jobs.get()
                if job is None:
                    return
                try:
                    self.done.put(job())
                except Exception as exc:      # surfaces in the lane's thread
                    self.done.put(exc)

        def close(self):
            self.jobs.put(None)
            self.thread.join()
            self.ctx2.close()
            if self.own_ctx:
                self.ctx.close()

    lanes = [Lane(ctx)] + [Lane(None) for _ in range(max(1, in_flight) - 1)]
    serial = len(lanes) == 1          # one step at a time: the flat commitment runs on the same stream as the rest
    hip = hip_event_timer()
    phases = {"encode": Events(hip), "commit": Events(hip), "tree": Events(hip), "open": Events(hip), "verify": Events(hip)}

    def quantise(lane):
        lane.ctx.quant_scale(dx, n, lane.scale)
        lane.ctx.encode_tensor_scaled(dx, T.TC_F16, n, lane.scale, lane.dq)

    quantise(lanes[0])
    ctx.sync()
    q = lanes[0].dq.cpu().numpy().reshape(shape)
    leaf_values = [(int(q[l]) % R_MODULUS).to_bytes(32, "little") for l in leaves]

    def step(record, lane=None):
        lane = lane or lanes[0]
        lctx, dq = lane.ctx, lane.dq

        def timed(name, fn):
            if not record:
                return fn()
            p = phases[name].start()
            out = fn()
            phases[name].stop(p)
            return out

        timed("encode", lambda: quantise(lane))
        if record or serial:
            C = timed("commit", lambda: lctx.commit(srs, dq, T.TC_I16))
            tree = timed("tree", lambda: lctx.terkle_build_entries(node_srs, dq, T.TC_I16, shape, node))
        else:
            lctx.sync()                                  # the quantised tensor is complete before the side stream reads it
            lane.jobs.put(lambda: lane.ctx2.commit(srs, dq, T.TC_I16))
            tree = lctx.terkle_build_entries(node_srs, dq, T.TC_I16, shape, node)
            C = None
        proofs = timed("open", lambda: tree.open_batch(leaves))
        root = tree.root
        ok = timed("verify", lambda: lctx.verify_paths_batch(vk, paths, [root] * len(leaves), leaf_values, proofs))
        tree.close()
        if C is None:                                    # the step ends when the flat commitment is in as well
            C = lane.done.get()
            if isinstance(C, Exception):
                raise C
        return C, root, ok

    def run_steps(count_per_lane):
        """Deals the steps out to the lanes, one host thread per lane; returns every step's results."""
        results, errors = [[] for _ in lanes], []

        def work(i):
            try:
                for _ in range(count_per_lane[i]):
                    results[i].append(step(False, lanes[i]))
            except Exception as exc:
                errors.append(exc)

        if len(lanes) == 1:
            work(0)
        else:
            threads = [threading.Thread(target=work, args=(i,)) for i in range(len(lanes)) if count_per_lane[i]]
            for t in threads:
                t.start()
            for t in threads:
                t.join()
        if errors:
            raise errors[0]
        return [r for lane_results in results for r in lane_results]

    def deal(total):
        return [total // len(lanes) + (1 if i < total % len(lanes) else 0) for i in range(len(lanes))]

    # priming, part of the untimed set-up: a fresh process on a fresh box needs more than a few steps before the
    # lanes overlap fully (workspaces grow to their final size, code objects load, clocks and host threads settle)
    PRIMING_STEPS = 12
    run_steps([PRIMING_STEPS] * len(lanes))
    run_steps([warmup] * len(lanes))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    timed_results = run_steps(deal(steps))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert len(timed_results) == steps
    assert all(all(r[2]) for r in timed_results), "path verification failed inside the benchmark"
    C_timed, root_timed = timed_results[0][0], timed_results[0][1]
    assert all(r[0] == C_timed and r[1] == root_timed for r in timed_results)
    # latency of one step on its own (lane 0, nothing else in flight)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(min(steps, 5)):
        step(False)
    torch.cuda.synchronize()
    step_latency_ms = (time.perf_counter() - t1) * 1e3 / min(steps, 5)
    # a second, serial pass with HIP events around every phase and around the long kernels
    for kind in range(4):
        ctx.profile_read(kind)
    ctx.profile_units(B.TC_PROF_BUCKET_ACC)
    ctx.profile(True)
    prof_steps = min(steps, 5)
    for _ in range(prof_steps):
        C, root, ok = step(True)
    torch.cuda.synchronize()
    assert C == C_timed and root == root_timed and all(ok)
    phase_ms = {k: v.total_ms() / prof_steps for k, v in phases.items()}
    nonzero = int(np.count_nonzero(q))
    acc_ms, acc_launches = ctx.profile_read(B.TC_PROF_BUCKET_ACC)
    acc_executed = ctx.profile_units(B.TC_PROF_BUCKET_ACC) / max(acc_launches, 1)
    node_ms, node_launches = ctx.profile_read(B.TC_PROF_NODE_COMMIT)
    upper_ms, upper_launches = ctx.profile_read(B.TC_PROF_NODE_COMMIT_UPPER)
    chain_ms, chain_launches = ctx.profile_read(B.TC_PROF_VERIFY_CHAIN)
    ctx.profile(False)
    kern_ms = acc_ms / max(acc_launches, 1)
    per_mixed = FP_MULS_PER_MIXED_ADD * MADS_PER_FP_MUL
    levels, g = [], shape
    while True:
        g = tuple(-(-d // b) for d, b in zip(g, node))
        levels.append(int(np.prod(g)))
        if all(d == 1 for d in g):
            break
    upper_children = sum(levels[:-1])

    def kernel_line(name, ms_step, mads_step, note):
        ach = mads_step / (ms_step * 1e-3) if ms_step > 0 else 0.0
        return {"kernel": name, "ms_per_step": ms_step, "achieved": ach / 1e12, "frac": ach / peak, "note": note}

    chains = sum(2 * int(p.m[s]) for p in paths for s in range(p.n_steps))
    out = {
        "workload": "C2: 512x4096 fp16 N(0,1) activation -> int16 (scale and quantisation on the device), one tensor commitment + "
                    "arity-16 (4,4) Terkle tree over 2^21 entries (139813 nodes) + %d path openings + verification" % openings,
        "elements": n, "steps": steps, "steps_in_flight": len(lanes), "priming_steps_per_lane_untimed": PRIMING_STEPS,
        "hw_queues": int(os.environ["GPU_MAX_HW_QUEUES"]),
        "elements_per_s": n * steps / elapsed, "ms_per_step": elapsed * 1e3 / steps, "step_latency_ms": step_latency_ms,
        "phase_ms_serial": phase_ms, "commit_only_elements_per_s": n / (phase_ms["commit"] * 1e-3),
        "kernels": [
            kernel_line("AccAffine (bucket accumulation of tc_commit)", kern_ms, acc_executed * per_mixed,
                        "%d of %d mixed additions run in this launch, the rest in the passes after it" % (acc_executed, nonzero)),
            kernel_line("NodeCommitSmall (level 0 of the tree)", node_ms / prof_steps, nonzero * per_mixed,
                        "one mixed addition per non-zero entry, fixed-base tables"),
            kernel_line("node commitments of levels 1..%d" % (len(levels) - 1), upper_ms / prof_steps,
                        upper_children * 16 * per_mixed, "16 window terms per child; %d launches a step, the small levels bound by depth" % (upper_launches // prof_steps)),
            kernel_line("VerifyChain", chain_ms / prof_steps, chains * 127 * 7 * MADS_PER_FP_MUL,
                        "%d chains of 127 Jacobian doublings, three waves a chain group: bound by depth" % chains),
        ],
    }
    # public verification of one of this step's paths with the pairing, on the host
    pv = B.PairingVerifier(tau, 2, lib)
    tree = ctx.terkle_build_entries(node_srs, lanes[0].dq, T.TC_I16, shape, node)
    proofs = tree.open_batch(leaves)
    t_pv = time.perf_counter()
    ok_pv = [pv.verify_path(p, tree.root, v, pr) for p, v, pr in zip(paths, leaf_values, proofs)]
    t_pv = (time.perf_counter() - t_pv) * 1e3 / len(paths)
    assert all(ok_pv)
    out["public_verification"] = {"ms_per_path": t_pv, "steps_per_path": int(paths[0].n_steps), "where": "host CPU, one thread",
                                  "how": "pairing form of Ver: the steps of a path combined with random weights into "
                                         "3 Miller loops and one final exponentiation"}
    tree.close()
    pv.close()
    for lane in lanes[1:]:
        lane.close()
    lanes[0].jobs.put(None)
    lanes[0].thread.join()
    lanes[0].ctx2.close()
    srs.close()
    return out, q


def encode_stream(ctx, T, torch):
    """the quantisation kernels on a tensor large enough to be bound by HBM rather than by the launch"""
    big_n = 1 << 28
    big_in = torch.randn(big_n, dtype=torch.float16, device="cuda")
    big_out = torch.empty(big_n, dtype=torch.int16, device="cuda")
    scale = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.encode_tensor(big_in.view(torch.int16), T.TC_F16, big_n, 1000.0, big_out)
    ctx.quant_scale(big_in.view(torch.int16), big_n, scale)
    ctx.sync()
    t0 = time.perf_counter()
    for _ in range(5):
        ctx.encode_tensor(big_in.view(torch.int16), T.TC_F16, big_n, 1000.0, big_out)
    ctx.sync()
    enc_ms = (time.perf_counter() - t0) * 1e3 / 5
    t0 = time.perf_counter()
    for _ in range(5):
        ctx.quant_scale(big_in.view(torch.int16), big_n, scale)
    ctx.sync()
    max_ms = (time.perf_counter() - t0) * 1e3 / 5
    return {"elements": big_n, "bound": "hbm", "peak": 8000.0, "unit": "GB/s",
            "encode": {"ms": enc_ms, "achieved": 4.0 * big_n / (enc_ms * 1e-3) / 1e9, "frac": 4.0 * big_n / (enc_ms * 1e-3) / 8e12,
                       "note": "tc_encode_tensor, fp16 -> int16: 2 bytes read and 2 bytes written per element"},
            "scale": {"ms": max_ms, "achieved": 2.0 * big_n / (max_ms * 1e-3) / 1e9, "frac": 2.0 * big_n / (max_ms * 1e-3) / 8e12,
                      "note": "tc_quant_scale: 2 bytes read per element"}}


def coefficient_route(ctx, T, torch, with_oracle, peak):
    """Interpolation to monomial coefficients (the first step of Com as Def. 4.1 prints it, bypassed by the hot
    path): the sweep of Fig. 1, N = 2^12 samples reshaped to order-m grids, in Newton form (`gpu_ms`) and in the
    Gregory and barycentric forms of App. C, and the C2 activation; one Fr product
    = 2 * 8^2 + 8 = 136 multiply-adds, an axis of length d costs 2 (d - 1) products per entry."""
    from oracle import tc as otc

    out = {"sweep_n_4096": []}
    rng = np.random.default_rng(5)
    for shape in ((4096,), (64, 64), (16, 16, 16), (8, 8, 8, 8), (4,) * 6, (2,) * 12):
        x = rng.integers(-32768, 32768, size=shape).astype(np.int16)
        dx = torch.from_numpy(x).cuda()
        coeffs = torch.empty(32 * x.size, dtype=torch.uint8, device="cuda")
        ctx.interpolate(shape, dx, T.TC_I16, coeffs)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            ctx.interpolate(shape, dx, T.TC_I16, coeffs)
        torch.cuda.synchronize()
        line = {"m": len(shape), "shape": list(shape), "gpu_ms": (time.perf_counter() - t0) * 1e3 / 3}
        for form, name in ((T.TC_INTERP_GREGORY, "gregory"), (T.TC_INTERP_BARYCENTRIC, "barycentric")):
            other = torch.empty_like(coeffs)
            ctx.interpolate_form(shape, dx, T.TC_I16, form, other)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(3):
                ctx.interpolate_form(shape, dx, T.TC_I16, form, other)
            torch.cuda.synchronize()
            line["gpu_ms_" + name] = (time.perf_counter() - t1) * 1e3 / 3
            assert torch.equal(other, coeffs), (shape, name)
        if with_oracle and len(shape) >= 2:
            t1 = time.perf_counter()
            want = otc.interpolate(x, shape)
            line["oracle_ms"] = (time.perf_counter() - t1) * 1e3
            raw = coeffs.cpu().numpy().tobytes()
            assert [int.from_bytes(raw[32 * i : 32 * (i + 1)], "little") for i in range(x.size)] == want
        out["sweep_n_4096"].append(line)
    shape = tc_inputs.C2_SHAPE
    x = tc_inputs.c2_activation()
    q = np.clip(np.rint(x.astype(np.float32) * 1000.0), -32767, 32767).astype(np.int16)
    dx = torch.from_numpy(q).cuda()
    coeffs = torch.empty(32 * q.size, dtype=torch.uint8, device="cuda")
    ctx.interpolate(shape, dx, T.TC_I16, coeffs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.interpolate(shape, dx, T.TC_I16, coeffs)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    mads = q.size * sum(2 * (d - 1) for d in shape) * 136
    out["c2_activation"] = {"shape": list(shape), "ms": ms, "achieved": mads / (ms * 1e-3) / 1e12,
                            "frac": mads / (ms * 1e-3) / peak, "unit": "T 32x32->64 multiply-add/s"}
    return out


def tree_scaling(ctx, T, torch, tau):
    """The tree-scaling comparison of Fig. 4 as a workload: arity B = 64, 64^1 .. 64^4 int16 leaves, Terkle node
    shapes (8,8) and (4,4,4) and the Verkle tree as node shape (64,): build, 8 openings in one batch, their
    batch verification on the GPU, public verification of one path on the host, one incremental update."""
    out = []
    vk = ctx.vk_from_trapdoor(tau)
    for node in ((8, 8), (4, 4, 4), (64,)):
        m = len(node)
        srs = ctx.setup_from_trapdoor(tau, node, T.TC_SRS_SUFFIX | T.TC_SRS_FIXED_BASE)
        pv = T.PairingVerifier(tau, m)
        for k in (1, 2, 3, 4):
            grid = tuple(d**k for d in node)
            n = 64**k
            x = tc_inputs.int16_uniform(grid, 100 + k)
            dx = torch.from_numpy(x).cuda()
            leaves = tc_inputs.opening_positions(grid, 8, 7)
            tree = ctx.terkle_build_entries(srs, dx, T.TC_I16, grid, node)
            tree.close()
            ctx.sync()

            def clock(fn, reps=3):
                best = None
                for _ in range(reps):
                    ctx.sync()
                    t0 = time.perf_counter()
                    r = fn()
                    ctx.sync()
                    dt = (time.perf_counter() - t0) * 1e3
                    best = dt if best is None or dt < best else best
                return best, r

            build_ms, tree = clock(lambda: ctx.terkle_build_entries(srs, dx, T.TC_I16, grid, node), 1)
            open_ms, proofs = clock(lambda: tree.open_batch(leaves))
            paths = [tree.path(l) for l in leaves]
            values = [(int(x[l]) % R_MODULUS).to_bytes(32, "little") for l in leaves]
            verify_ms, ok = clock(lambda: ctx.verify_paths_batch(vk, paths, [tree.root] * 8, values, proofs))
            assert all(ok)
            t0 = time.perf_counter()
            assert pv.verify_path(paths[0], tree.root, values[0], proofs[0])
            public_ms = (time.perf_counter() - t0) * 1e3
            root_before = tree.root
            update_ms, _ = clock(lambda: tree.update(leaves[0], 1), 1)
            assert tree.root != root_before
            tree.update(leaves[0], -1)
            assert tree.root == root_before
            out.append({"node_shape": list(node), "leaves": n, "levels": tree.levels, "build_ms": build_ms,
                        "open_8_paths_ms": open_ms, "verify_8_paths_gpu_ms": verify_ms, "verify_1_path_pairing_cpu_ms": public_ms,
                        "update_1_entry_ms": update_ms})
            tree.close()
            del dx
        pv.close()
        srs.close()
    return out


def other_configs(ctx, T, torch, node_srs, tau):
    """Configurations 4 and 5 at their stated sizes, timed once each (their parity is the GPU tests' business):
    the int8 weight matrices of all 32 LLaMA2-7B-shaped layers committed and put under one tree, and the eight
    LLaMA2-13B-shaped requests -- quantise, build, 128 path openings each, then all 1024 paths verified in one batch."""
    out = {}
    # ---- config 4
    shapes7 = tc_inputs.c4_shapes()
    srs4 = {s: ctx.setup_from_trapdoor(tau, s, 0) for s in set(shapes7)}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(tc_inputs.tensor_seed(3))
    layers = tc_inputs.LLAMA7B["layers"]
    leaves = [torch.randint(-127, 128, (s[0] * s[1],), generator=gen, device="cuda", dtype=torch.int8) for _ in range(layers) for s in shapes7]
    leaf_srs = [srs4[s] for _ in range(layers) for s in shapes7]
    scalars = sum(x.numel() for x in leaves)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tree = ctx.terkle_build_tensors(node_srs, leaf_srs, leaves, [T.TC_I8] * len(leaves), (layers, 7), tc_inputs.NODE_SHAPE)
    ms = (time.perf_counter() - t0) * 1e3
    assert len(tree.root) == 96
    tree.close()
    out["c4_weights"] = {"workload": "C4: 32 layers x 7 LLaMA2-7B-shaped weight matrices, int8 uniform in [-127, 127], "
                                     "224 commitments and the (4,4) tree over them in one tc_terkle_build",
                         "scalars": scalars, "ms": ms, "scalars_per_s": scalars / (ms * 1e-3)}
    del leaves, leaf_srs
    for s in srs4.values():
        s.close()
    # ---- config 5
    cfg = tc_inputs.LLAMA13B
    shapes3 = tc_inputs.c3_shapes(cfg)
    srs5 = {s: ctx.setup_from_trapdoor(tau, s, T.TC_SRS_SUFFIX | T.TC_SRS_OPEN_TABLE) for s in set(shapes3)}
    vk = ctx.vk_from_trapdoor(tau)
    grid = (cfg["layers"], 3)
    gen.manual_seed(tc_inputs.tensor_seed(4))
    rng = np.random.default_rng(tc_inputs.tensor_seed(4) + 999)
    n_leaves = grid[0] * 3
    qs = [torch.empty(shapes3[i % 3][0] * shapes3[i % 3][1], dtype=torch.int16, device="cuda") for i in range(n_leaves)]
    scales = torch.zeros(n_leaves, dtype=torch.float32, device="cuda")
    leaf_srs = [srs5[shapes3[i % 3]] for i in range(n_leaves)]
    elements = sum(q.numel() for q in qs)
    quant_ms, build_ms, open_ms = [], [], []
    paths, roots, values, proofs = [], [], [], []
    for _req in range(cfg["batch"]):
        xs = [torch.randn(q.numel(), generator=gen, device="cuda", dtype=torch.float32).to(torch.float16) for q in qs]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.encode_batch_scaled(xs, [x.numel() for x in xs], scales, qs)
        ctx.sync()
        t1 = time.perf_counter()
        tree = ctx.terkle_build_tensors(node_srs, leaf_srs, qs, [T.TC_I16] * n_leaves, grid, tc_inputs.NODE_SHAPE)
        t2 = time.perf_counter()
        del xs
        where = [(int(rng.integers(0, grid[0])), int(rng.integers(0, 3))) for _ in range(128)]
        inner = [tuple(int(rng.integers(0, d)) for d in shapes3[l[1]]) for l in where]
        t3 = time.perf_counter()
        got = tree.open_batch(where, inner)
        t4 = time.perf_counter()
        flat = torch.stack([qs[l[0] * 3 + l[1]][i[0] * shapes3[l[1]][1] + i[1]] for l, i in zip(where, inner)])
        values += [(int(v) % R_MODULUS).to_bytes(32, "little") for v in flat.cpu().tolist()]
        paths += [tree.path(l, i) for l, i in zip(where, inner)]
        roots += [tree.root] * 128
        proofs += got
        quant_ms.append((t1 - t0) * 1e3)
        build_ms.append((t2 - t1) * 1e3)
        open_ms.append((t4 - t3) * 1e3)
        tree.close()
    t0 = time.perf_counter()
    ok = ctx.verify_paths_batch(vk, paths, roots, values, proofs)
    verify_ms = (time.perf_counter() - t0) * 1e3
    assert all(ok), "C5 openings failed verification"
    assert len(set(roots)) == cfg["batch"]
    med = lambda v: sorted(v)[len(v) // 2]
    out["c5_batched_requests"] = {
        "workload": "C5: 8 LLaMA2-13B-shaped requests, each 40 layers x {2048x5120, 2048x5120, 2048x13824} fp16 N(0,1) -> int16, "
                    "one (4,4) tree per request, 128 random path openings per request, the 1024 paths verified in one batch",
        "elements_per_request": elements, "requests": cfg["batch"],
        "quantise_ms_per_request": med(quant_ms), "build_ms_per_request": med(build_ms),
        "build_elements_per_s": elements / (med(build_ms) * 1e-3),
        "open_128_paths_ms_per_request": med(open_ms), "verify_1024_paths_ms": verify_ms}
    for s in srs5.values():
        s.close()
    return out


def layer_selection(T, lib, with_oracle):
    """the verifier's layer selection (Problem 4.5) on synthetic benefits: library O(M L) against the oracle's O(M L^2)"""
    rng_sel = np.random.default_rng(9)
    Lsel, Msel = 2000, 8
    nu_s, phi_s = (rng_sel.random(Lsel) ** 3).tolist(), (1.0 + rng_sel.random(Lsel)).tolist()
    beta_s = (50.0 + 50.0 * rng_sel.random(Msel)).tolist()
    t0 = time.perf_counter()
    T.binding.select_layers(nu_s, phi_s, beta_s, lib)
    sel_ms = (time.perf_counter() - t0) * 1e3
    out = {"layers": Lsel, "verifiers": Msel, "ms": sel_ms, "where": "host CPU, one thread (incl. marshalling)"}
    if with_oracle:
        from oracle import selector as osel
        t0 = time.perf_counter()
        table = osel.dp_naive(nu_s[:400], phi_s[:400], beta_s)
        out["oracle_ms_400_layers"] = (time.perf_counter() - t0) * 1e3
        v400, _ = T.binding.select_layers(nu_s[:400], phi_s[:400], beta_s, lib)
        assert abs(v400 - table[Msel][400]) <= 1e-9 * max(1.0, abs(v400))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--lib", default=None, help="path of an alternative libtc.so (experiments)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-c2", action="store_true", help="skip the single-layer step with steps in flight (sub-object c2_step)")
    ap.add_argument("--no-extras", action="store_true", help="skip the sub-objects beyond the hot path (coefficient route, layer selection, encode stream)")
    ap.add_argument("--no-configs", action="store_true", help="skip the one-off timings of configurations 4 and 5 at their stated sizes "
                    "(sub-objects c4_weights, c5_batched_requests; about 40 GB of device memory and 25 s)")
    ap.add_argument("--c2-steps", type=int, default=60, help="timed steps of the c2_step leg")
    ap.add_argument("--openings", type=int, default=8, help="path openings per step of the c2_step leg")
    ap.add_argument("--in-flight", type=int, default=12, help="steps in flight of the c2_step leg: each has its own host thread, "
                    "contexts, streams and buffers (1 = one step after the other)")
    ap.add_argument("--fig4", action="store_true", help="also run the arity-64 tree-scaling workload (64^1 .. 64^4 leaves, "
                    "node shapes (8,8), (4,4,4), (64,)); needs about 12 GB of fixed-base tables")
    ap.add_argument("--only-c3-build", type=int, default=0, metavar="N", help="profiling mode: set-up, N quantise + build "
                    "passes of the LLaMA2-7B-shaped forward, nothing else")
    ap.add_argument("--only-c2-step", action="store_true", help="profiling mode: set-up and the single-layer leg alone "
                    "(--c2-steps, --in-flight; --in-flight 1 runs one step after the other)")
    ap.add_argument("--calibrate-copy", action="store_true", help="also run one plain copy kernel of 256 MiB "
                    "(reference dispatch for scaling the HBM byte counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2602_12630_amd as T

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    lib = T.load_library(args.lib) if args.lib else None
    ctx = T.Context(0, None, lib)
    tau = tc_inputs.trapdoor_bytes()
    node = tc_inputs.NODE_SHAPE

    t0 = time.time()
    node_srs = ctx.setup_from_trapdoor(tau, node, T.TC_SRS_SUFFIX | T.TC_SRS_FIXED_BASE)
    ctx.sync()
    setup_s = time.time() - t0

    if args.calibrate_copy:
        cal_src = torch.zeros(128 * 1024 * 1024, dtype=torch.int16, device="cuda")
        cal_dst = torch.empty_like(cal_src)
        ctx.encode_tensor(cal_src, T.TC_I16, cal_src.numel(), 1.0, cal_dst)      # Copy128: 256 MiB read, 256 MiB written
        ctx.sync()
        del cal_src, cal_dst
    if args.only_c3_build:
        only_c3_build(ctx, T, torch, node_srs, tau, args.only_c3_build)
        node_srs.close()
        ctx.close()
        return
    if args.only_c2_step:
        leg, _ = bench_c2_step(ctx, T, torch, lib, node_srs, tau, args.c2_steps, max(args.warmup, 2), args.in_flight, args.openings,
                               FORMULA_PEAK_MADS_PER_S)
        print(json.dumps({"mode": "only-c2-step", "c2_step": leg}))
        node_srs.close()
        ctx.close()
        return

    peak_obj = alu_peak(ctx, T)
    peak = peak_obj["used"]
    c3 = bench_c3(ctx, T, torch, node_srs, tau, args.steps, args.warmup, peak)
    out = {
        "metric": "tensor elements committed/sec",
        "value": c3.pop("value"),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": c3.pop("ms_per_step"),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": "C3: LLaMA2-7B-shaped forward, 32 layers x {512x4096, 512x4096, 512x11008} fp16 N(0,1) -> int16 "
                               "(scale and quantisation on the device), 96 tensor commitments, arity-16 (4,4) Terkle tree over "
                               "them, 64 random path openings down to tensor entries, batch verification; one stream",
                   "elements": c3.pop("elements"), "node_srs_setup_s_untimed": setup_s},
        "terkle_build_ms_per_llama2_7b_fwd": c3.pop("terkle_build_ms_per_llama2_7b_fwd"),
        "build_elements_per_s": c3.pop("build_elements_per_s"),
        "roofline": c3.pop("roofline"),
        "alu_peak": peak_obj,
    }
    out.update(c3)
    q = None
    if not args.no_c2:
        out["c2_step"], q = bench_c2_step(ctx, T, torch, lib, node_srs, tau, args.c2_steps, max(args.warmup, 2), args.in_flight,
                                          args.openings, peak)
    if not args.no_extras:
        out["encode_stream"] = encode_stream(ctx, T, torch)
        out["layer_selection"] = layer_selection(T, lib, not args.no_cpu_baseline)
        out["coefficient_route"] = coefficient_route(ctx, T, torch, not args.no_cpu_baseline, peak)
    if not args.no_configs:
        out.update(other_configs(ctx, T, torch, node_srs, tau))
    if args.fig4:
        out["tree_scaling"] = tree_scaling(ctx, T, torch, tau)
    if not args.no_cpu_baseline:
        if q is None:
            from oracle import quantize
            x = tc_inputs.c2_activation()
            q = quantize.quantize_f16(x, quantize.inv_scale_for(x))
        out["cpu_baseline"] = cpu_baseline(q)
    print(json.dumps(out))
    node_srs.close()
    ctx.close()


if __name__ == "__main__":
    main()
