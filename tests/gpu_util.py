"""Helpers shared by the GPU parity tests: device buffers through torch, oracle-side caches."""
import os
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import tc_inputs
from oracle import bls12_381 as ec
from oracle import cbind, tc

TAU = tc_inputs.trapdoors()
TAU_BYTES = tc_inputs.trapdoor_bytes()
_pp = {}


def pps(shape):
    shape = tuple(int(d) for d in shape)
    if shape not in _pp:
        _pp[shape] = tc.setup(shape, TAU)
    return _pp[shape]


def to_device(arr):
    import torch

    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def fr_bytes_array(values):
    """Python ints -> contiguous uint8 array of canonical 32-byte Fr values."""
    return np.frombuffer(b"".join(ec.fr_to_bytes(int(v) % ec.R) for v in values), dtype=np.uint8).copy()


def serialize_steps(steps):
    """Oracle path steps -> the proof byte layout of the library (top level first)."""
    out = b""
    for i, (_k, y, pi, child) in enumerate(steps):
        out += b"".join(ec.g1_to_bytes(p) for p in pi) + ec.fr_to_bytes(y)
        if i + 1 < len(steps):                    # every step but the last carries the next commitment (may be the identity)
            out += ec.g1_to_bytes(child)
    return out


def parse_proof(path, proof):
    """Library proof bytes -> oracle path steps (kappa, y, [pi], child) and the step shapes, top first."""
    steps, shapes, off = [], [], 0
    for s in range(path.n_steps):
        m = path.m[s]
        pi = [ec.g1_from_bytes(proof[off + 96 * i : off + 96 * (i + 1)]) for i in range(m)]
        off += 96 * m
        y = ec.fr_from_bytes(proof[off : off + 32])
        off += 32
        child = None
        if s < path.n_steps - 1:
            child = ec.g1_from_bytes(proof[off : off + 96])
            off += 96
        steps.append((tuple(path.kappa[s][j] for j in range(m)), y, pi, child))
        shapes.append(tuple(path.shape[s][j] for j in range(m)))
    assert off == len(proof)
    return steps, shapes


# ---- oracle work on all host cores --------------------------------------------------------------------
# numpy's generators and ufuncs and the C oracle (through ctypes) all release the interpreter lock, so a pool of
# threads keeps the machine's cores busy; the GPU machine gives a test 16 of them whatever os.cpu_count() says.
HOST_THREADS = min(16, os.cpu_count() or 1)


def oracle_pool():
    cbind.lib()                                    # load the C oracle before several threads ask for it
    return ThreadPoolExecutor(max_workers=HOST_THREADS)


CAPTURE_MANAGER = None      # pytest's capture manager, set by conftest.py


def progress(line):
    """One line to the real stdout, whether or not pytest is capturing output."""
    if CAPTURE_MANAGER is not None:
        with CAPTURE_MANAGER.global_and_fixture_disabled():
            print(line, flush=True)
    else:
        print(line, flush=True)


class Stopwatch:
    """Prints what a long test is doing and how long each part took (the GPU machine takes silence for a hang)."""

    def __init__(self, name):
        self.name, self.t0, self.last = name, time.time(), time.time()

    def lap(self, what):
        now = time.time()
        progress("%s: %s (%.1f s, %.1f s since start)" % (self.name, what, now - self.last, now - self.t0))
        self.last = now


def check_field_arithmetic(run, n_fp, n_fr):
    """run(op, a_words, b_words, words_per_element) -> result words, for the operations of tc_ctx_field_op; every
    result is compared with Python integers.  Operands are Montgomery representatives, i.e. plain residues."""
    import random

    P, Rr = ec.P, ec.R
    RP, RR = 1 << 384, 1 << 256
    rng = random.Random(11)
    edge_p = [0, 1, 2, P - 1, P - 2, 1 << 380, (1 << 380) - 1, RP % P, (RP * RP) % P, (1 << 381) % P,
              int("ffffffff" * 11, 16), 0xFFFFFFFF, 1 << 32, (P - 1) // 2, (P + 1) // 2]
    a_vals = edge_p + [rng.randrange(P) for _ in range(n_fp)] + [x for x in edge_p for _ in edge_p]
    b_vals = list(reversed(edge_p)) + [rng.randrange(P) for _ in range(n_fp)] + [y for _ in edge_p for y in edge_p]

    def pack(vals, words):
        return np.frombuffer(b"".join(int(v).to_bytes(4 * words, "little") for v in vals), dtype=np.uint32).copy()

    def unpack(arr, words):
        raw = np.ascontiguousarray(arr).tobytes()
        return [int.from_bytes(raw[4 * words * i : 4 * words * (i + 1)], "little") for i in range(len(raw) // (4 * words))]

    pa, pb = pack(a_vals, 12), pack(b_vals, 12)
    rinv = pow(RP, -1, P)
    expect = {0: lambda x, y: x * y * rinv % P, 1: lambda x, y: x * x * rinv % P, 2: lambda x, y: x * y * rinv % P,
              3: lambda x, y: x * x * rinv % P, 6: lambda x, y: (x + y) % P, 7: lambda x, y: (x - y) % P,
              # the 28-bit-limb form of the bucket accumulation: unreduced sums and differences with signed limbs
              9: lambda x, y: x * y * rinv % P, 10: lambda x, y: x * x * rinv % P,
              11: lambda x, y: (x - y) * (x + y) * rinv % P, 12: lambda x, y: (x - 2 * y) * (x - y) * rinv % P,
              13: lambda x, y: (x - y) * x * rinv % P}
    for op, fn in expect.items():
        got = unpack(run(op, pa, pb, 12), 12)
        bad = [i for i in range(len(a_vals)) if got[i] != fn(a_vals[i], b_vals[i])]
        assert not bad, "Fp operation %d: %d wrong, first operands %x, %x" % (op, len(bad), a_vals[bad[0]], b_vals[bad[0]])
    nz = [v if v else 5 for v in a_vals]                       # inverse of a Montgomery representative: R^2 / a
    got = unpack(run(4, pack(nz, 12), pack(nz, 12), 12), 12)
    assert all(g == RP * RP * pow(v, -1, P) % P for g, v in zip(got, nz)), "Fp inverse"
    edge_r = [0, 1, Rr - 1, RR % Rr, 1 << 254, (1 << 254) - 1, 0xFFFFFFFF]
    ar = edge_r + [rng.randrange(Rr) for _ in range(n_fr)] + [x for x in edge_r for _ in edge_r]
    br = list(reversed(edge_r)) + [rng.randrange(Rr) for _ in range(n_fr)] + [y for _ in edge_r for y in edge_r]
    rrinv = pow(RR, -1, Rr)
    got = unpack(run(5, pack(ar, 8), pack(br, 8), 8), 8)
    assert all(g == x * y * rrinv % Rr for g, x, y in zip(got, ar, br)), "Fr product"
    nzr = [v if v else 7 for v in ar]
    got = unpack(run(8, pack(nzr, 8), pack(nzr, 8), 8), 8)
    assert all(g == RR * RR * pow(v, -1, Rr) % Rr for g, v in zip(got, nzr)), "Fr inverse"


def check_one_point_throughout(ctx, upload, shape):
    """Public parameters that are one and the same point at every position, at a size whose passes over the partial
    sums fill the chip: every addition in them is a doubling or a cancellation, so every lane of the fast passes
    gives up and the second launches redo them.  sum_i v_i P = [sum_i v_i] P."""
    import paper_2602_12630_amd as T

    n = int(np.prod(shape))
    srs = ctx.setup_from_trapdoor(TAU_BYTES, (2, 2), 0)
    pt = srs.point(3)
    srs.close()
    big = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    header = bytes(big.export()[:56])
    big.close()
    back = ctx.srs_import(header + pt * n)
    P = ec.g1_from_bytes(pt)
    nrng = np.random.default_rng(17)
    for X, dtype in ((nrng.integers(-100, 101, size=shape).astype(np.int8), T.TC_I8),
                     (nrng.integers(-3, 4, size=shape).astype(np.int16), T.TC_I16)):
        total = int(X.astype(np.int64).sum())
        want = ec.mul(total % ec.R, P)
        assert ctx.commit(back, upload(X), dtype) == ec.g1_to_bytes(want), dtype
    back.close()


def check_repeated_points(ctx, upload, many=512):
    """Commitments over public parameters in which most points repeat or are each other's negatives, with scalars of
    few distinct values: the bucket sums then run into doublings, sums that cancel to the identity and additions to
    the identity, the cases that the accumulation kernel's fast form of the chord rule hands to the slower routine.
    Then the same in batches: eight int16 tensors in one call (the row and column sums of their 128 x 256 bucket
    matrices go one lane per piece, with a list for the sums that meet equal or opposite points) and `many` int8
    tensors in one call (that many windows of 128 buckets, a lane per row and column).
    Expected values: the C oracle's term-by-term sum over the same points.  `upload` puts a numpy array where the
    context reads it (device memory, or the array itself on the host build)."""
    import random

    import paper_2602_12630_amd as T

    shape = (32, 128)
    n = 32 * 128
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    data = bytes(srs.export())
    srs.close()
    assert len(data) == 56 + 96 * n
    pts = [data[56 + 96 * i : 56 + 96 * (i + 1)] for i in range(n)]

    def neg(pt):
        return pt[:48] + ((ec.P - int.from_bytes(pt[48:], "little")) % ec.P).to_bytes(48, "little")

    rng = random.Random(5)
    pool = pts[:6]
    mixed = []
    for i in range(n):
        if rng.random() < 0.25:
            mixed.append(pts[i])
        else:
            q = pool[rng.randrange(len(pool))]
            mixed.append(q if rng.random() < 0.5 else neg(q))
    same = [pts[0]] * n                                     # one point throughout: every addition is a doubling or a cancellation
    nrng = np.random.default_rng(9)
    cases = [
        (mixed, nrng.integers(-3, 4, size=shape).astype(np.int8), T.TC_I8),
        (mixed, nrng.choice(np.array([-700, -5, 5, 9, 700], np.int16), size=shape), T.TC_I16),
        (mixed, nrng.integers(-32768, 32768, size=shape).astype(np.int16), T.TC_I16),
        (same, nrng.integers(-2, 3, size=shape).astype(np.int8), T.TC_I8),
        (same, np.full(shape, 77, np.int16), T.TC_I16),
        (same, np.where(nrng.random(shape) < 0.5, 1, -1).astype(np.int8), T.TC_I8),
    ]
    for points, X, dtype in cases:
        blob = b"".join(points)
        back = ctx.srs_import(data[:56] + blob)
        want, _ = cbind.msm_naive(X, blob, HOST_THREADS)
        got = ctx.commit(back, upload(X), dtype)
        back.close()
        assert got == ec.g1_to_bytes(want), (dtype, X.reshape(-1)[:8])
    for points in (mixed, same):
        blob = b"".join(points)
        back = ctx.srs_import(data[:56] + blob)
        X16 = [nrng.choice(np.array([-700, -5, 5, 9, 700], np.int16), size=shape) for _ in range(8)]
        X16[3] = np.full(shape, 9, np.int16)
        X8 = [nrng.integers(-3, 4, size=shape).astype(np.int8) for _ in range(many)]
        X8[1] = np.full(shape, -2, np.int8)
        for batch, dtype in ((X16, T.TC_I16), (X8, T.TC_I8)):
            held = [upload(X) for X in batch]
            got = ctx.commit_batch([back] * len(batch), held, [dtype] * len(batch))
            for j, X in enumerate(batch):
                want, _ = cbind.msm_naive(X, blob, HOST_THREADS)
                assert got[j] == ec.g1_to_bytes(want), (dtype, j)
        back.close()
