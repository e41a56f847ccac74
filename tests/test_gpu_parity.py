"""GPU parity: the HIP library through its C ABI against the CPU oracle, byte for byte.

All integer work, so every comparison is exact equality of canonical encodings."""
import json
import os

import numpy as np
import pytest

import tc_inputs
from oracle import bls12_381 as ec
from oracle import cbind, quantize, tc, terkle
from oracle.bls12_381 import R

from gpu_util import HOST_THREADS, TAU_BYTES, Stopwatch, check_field_arithmetic, check_one_point_throughout, check_repeated_points, fr_bytes_array, oracle_pool, parse_proof, pps, progress, serialize_steps, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import paper_2602_12630_amd as pkg

    return pkg


@pytest.fixture(scope="module")
def ctx(T):
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = T.Context(0)
    yield c
    c.close()


@pytest.fixture(scope="module")
def node_srs(T, ctx):
    s = ctx.setup_from_trapdoor(TAU_BYTES, tc_inputs.NODE_SHAPE, T.TC_SRS_SUFFIX | T.TC_SRS_FIXED_BASE)
    yield s
    s.close()


@pytest.fixture(scope="module")
def c1(T, ctx):
    srs = ctx.setup_from_trapdoor(TAU_BYTES, tc_inputs.C1_SHAPE, T.TC_SRS_SUFFIX)
    X = tc_inputs.c1_tensor()
    yield srs, X, to_device(X)
    srs.close()


def test_device_field_arithmetic_against_integers(T, ctx):
    """The device forms of the field arithmetic -- the product-scanning Montgomery product and square with inline
    multiply-add / carry instructions, their exact FP64-pipe variants, the word-batched binary-GCD inverse, the
    carry-chain addition and subtraction -- against Python integers, on edge operands (0, 1, p - 1, 2^380, the
    Montgomery one, all-ones limbs below p, every pair of them) and a few thousand random ones."""
    import torch

    def run(op, a, b, words):
        da, db = to_device(a), to_device(b)
        out = torch.empty(a.size, dtype=torch.int32, device="cuda")
        ctx.field_op(op, da, db, a.size // words, out)
        ctx.sync()
        return out.cpu().numpy().view(np.uint32)

    check_field_arithmetic(run, 4096, 1024)


def test_options_do_not_change_results(T, ctx):
    """The same int16 and full-width commitments under several plans of the accumulation (entries per lane, fan-in of
    the later passes, window width), with the on-curve guard switched on; the int16 one against the oracle."""
    B = T.binding
    shape = (64, 512)
    pp = pps(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    X = tc_inputs.int16_uniform(shape, 21, -32768, 32767)
    X.reshape(-1)[:5000] = 5
    F = fr_bytes_array([(v * 0x1F3D5B79A2C4E6F1) % R for v in range(1, 64 * 512 + 1)])
    dX, dF = to_device(X), to_device(F)
    want16 = ec.g1_to_bytes(cbind.commit(pp, X, HOST_THREADS))
    wantfr = None
    try:
        for sub, fan, win in ((0, 0, 0), (1, 2, 8), (3, 5, 16), (64, 64, 0)):
            ctx.set_option(B.TC_OPT_ACC_SUBRUN, sub)
            ctx.set_option(B.TC_OPT_ACC_FANIN, fan)
            ctx.set_option(B.TC_OPT_FR_WINDOW, win)
            ctx.set_option(B.TC_OPT_CHECK_LEVEL, 1)
            assert ctx.commit(srs, dX, T.TC_I16) == want16, (sub, fan, win)
            got = ctx.commit(srs, dF, T.TC_FR)
            wantfr = wantfr or got
            assert got == wantfr, (sub, fan, win)
    finally:
        for o in range(4):
            ctx.set_option(o, 0)
        srs.close()


def test_commit_over_repeated_points(ctx):
    """Equal and opposite points inside the bucket sums: the sub-runs that the fast accumulation gives up and the
    second launch redoes with every case of the group law (see check_repeated_points)."""
    check_repeated_points(ctx, to_device)


def test_commit_over_one_point_at_size(ctx):
    """The same at 2^21 terms, where the passes over the partial sums take their chip-filling kernels: one point at
    every position sends every lane of those passes to their second launch."""
    check_one_point_throughout(ctx, to_device, (512, 4096))


def test_srs_points_match_oracle(ctx, c1):
    srs, _, _ = c1
    pp = pps(tc_inputs.C1_SHAPE)
    rng = np.random.default_rng(1)
    for f in [0, 1023] + [int(v) for v in rng.integers(0, 1024, 10)]:
        want = ec.mul(pp.lagrange_scalar(tc.multi_index(f, pp.shape)), ec.G1)
        assert srs.point(f) == ec.g1_to_bytes(want)
    for a, n in ((1, 256), (2, 16)):
        assert srs.size(a) == n
        for f in (0, n - 1, n // 3):
            want = ec.mul(pp.lagrange_scalar(tc.multi_index(f, pp.shape[a:]), a), ec.G1)
            assert srs.point(f, a) == ec.g1_to_bytes(want)


def test_c1_commit_and_golden(T, ctx, c1):
    srs, X, dX = c1
    got = ctx.commit(srs, dX, T.TC_I8)
    assert got == ec.g1_to_bytes(tc.commit(pps(tc_inputs.C1_SHAPE), X))
    with open(os.path.join(os.path.dirname(__file__), "golden", "c1_oracle.json")) as f:
        gold = json.load(f)
    assert got.hex() == gold["commitment"]


def test_c1_openings_and_verification(T, ctx, c1):
    srs, X, dX = c1
    pp = pps(tc_inputs.C1_SHAPE)
    C = ctx.commit(srs, dX, T.TC_I8)
    vk = ctx.vk_from_trapdoor(TAU_BYTES)
    for kappa in tc_inputs.opening_positions(tc_inputs.C1_SHAPE, 8, tc_inputs.tensor_seed(0)):
        y, pi = ctx.open(srs, dX, T.TC_I8, kappa)
        yo, po = tc.open_(pp, X, kappa)
        assert y == ec.fr_to_bytes(yo)
        assert pi == [ec.g1_to_bytes(p) for p in po]
        assert ctx.verify(vk, tc_inputs.C1_SHAPE, C, kappa, y, pi)
        assert tc.verify(pp, ec.g1_from_bytes(C), kappa, yo, [ec.g1_from_bytes(p) for p in pi])
        assert not ctx.verify(vk, tc_inputs.C1_SHAPE, C, kappa, ec.fr_to_bytes((yo + 1) % R), pi)
        bad = list(pi)
        bad[1] = ec.g1_to_bytes(ec.add(po[1], ec.G1))
        assert not ctx.verify(vk, tc_inputs.C1_SHAPE, C, kappa, y, bad)


@pytest.mark.parametrize("shape", [(1,), (5,), (3, 4), (2, 3, 2), (2, 2, 2, 2), (7, 33), (16, 16)])
def test_commit_small_shapes_all_dtypes(T, ctx, shape):
    pp = pps(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    try:
        X16 = tc_inputs.int16_uniform(shape, 11, -32768, 32767)
        X16.reshape(-1)[0] = -32768
        X8 = tc_inputs.int8_uniform(shape, 12)
        X8.reshape(-1)[-1] = -128
        rng = np.random.default_rng(13)
        fr_vals = [int.from_bytes(rng.bytes(32), "little") % R for _ in range(tc.prod(shape))]
        assert ctx.commit(srs, to_device(X16), T.TC_I16) == ec.g1_to_bytes(tc.commit(pp, X16))
        assert ctx.commit(srs, to_device(X8), T.TC_I8) == ec.g1_to_bytes(tc.commit(pp, X8))
        assert ctx.commit(srs, to_device(fr_bytes_array(fr_vals)), T.TC_FR) == ec.g1_to_bytes(tc.commit(pp, fr_vals))
        kappa = tuple(d - 1 for d in shape)
        y, pi = ctx.open(srs, to_device(X16), T.TC_I16, kappa)
        yo, po = tc.open_(pp, X16, kappa)
        assert (y, pi) == (ec.fr_to_bytes(yo), [ec.g1_to_bytes(p) for p in po])
    finally:
        srs.close()


def test_special_tensors(T, ctx):
    shape = (6, 50)
    pp = pps(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    try:
        assert ctx.commit(srs, to_device(np.zeros(shape, np.int16)), T.TC_I16) == bytes(96)
        for c in (1, -1, 77, -32768, 32767):
            got = ctx.commit(srs, to_device(np.full(shape, c, np.int16)), T.TC_I16)
            assert got == ec.g1_to_bytes(ec.mul(c % R, ec.G1))                    # constant tensor => [c]G
        for f in (0, 149, 299):
            onehot = np.zeros(300, np.int8)
            onehot[f] = 1
            assert ctx.commit(srs, to_device(onehot), T.TC_I8) == srs.point(f)     # one-hot => S[f]
            onehot[f] = -1
            neg = ec.neg(ec.g1_from_bytes(srs.point(f)))
            assert ctx.commit(srs, to_device(onehot), T.TC_I8) == ec.g1_to_bytes(neg)
        # two entries that cancel: P + (-P)
        two = np.zeros(300, np.int16)
        two[5], two[6] = 9, -9
        want = ec.mul(9 * (pp.lagrange_scalar((0, 5)) - pp.lagrange_scalar((0, 6))) % R, ec.G1)
        assert ctx.commit(srs, to_device(two), T.TC_I16) == ec.g1_to_bytes(want)
    finally:
        srs.close()


def test_scalars_at_any_alignment(T, ctx):
    """The count / scatter kernels read sixteen bytes of scalars per lane where a tile starts on a 16-byte boundary
    and fall back to single values elsewhere: the same tensor at byte offsets 0, 2, 6 and 16 (int16) and 0, 1, 5
    (int8) of a device buffer, and a length that is no multiple of the chunk, against the oracle."""
    import torch

    shape = (61, 97)                                   # 5917 terms: tiles of 32 terms, ragged last tile
    n = shape[0] * shape[1]
    pp = pps(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    try:
        X16 = tc_inputs.int16_uniform(shape, 71, -32768, 32767)
        X8 = tc_inputs.int8_uniform(shape, 72)
        want16 = ec.g1_to_bytes(cbind.commit(pp, X16, nthreads=8))
        want8 = ec.g1_to_bytes(cbind.commit(pp, X8, nthreads=8))
        for off in (0, 1, 3, 8):
            buf = torch.zeros(n + 16, dtype=torch.int16, device="cuda")
            buf[off : off + n] = torch.from_numpy(X16.reshape(-1)).cuda()
            assert ctx.commit(srs, buf[off : off + n], T.TC_I16) == want16, off
        for off in (0, 1, 5):
            buf = torch.zeros(n + 16, dtype=torch.int8, device="cuda")
            buf[off : off + n] = torch.from_numpy(X8.reshape(-1)).cuda()
            assert ctx.commit(srs, buf[off : off + n], T.TC_I8) == want8, off
    finally:
        srs.close()


def test_degenerate_bucket_loads_at_size(T, ctx):
    """All terms in one bucket (constant tensor) and two-valued tensors at a size where the engine
    needs its shrinking passes; closed forms: constant c => [c]G, and linearity for the two-valued one."""
    shape = (512, 512)
    pp = pps(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    try:
        for c in (7, -32768):
            got = ctx.commit(srs, to_device(np.full(shape, c, np.int16)), T.TC_I16)
            assert got == ec.g1_to_bytes(ec.mul(c % R, ec.G1))
        X = np.full(shape, 3, np.int8)
        X[::2, :] = -5
        assert ctx.commit(srs, to_device(X), T.TC_I8) == ec.g1_to_bytes(cbind.commit(pp, X, nthreads=8))
    finally:
        srs.close()


def test_degenerate_bucket_loads_in_ordered_launches(T, ctx):
    """The same at 2^26 entries, where the accumulation hands its sub-runs out in the order of their lengths: a
    constant tensor (one bucket with a million sub-runs, all placed by one workgroup), and a tensor whose upper half is
    constant and whose lower half is Gaussian (one such bucket among ordinary ones), against the oracle's closed form."""
    shape = (8192, 8192)
    pp = pps(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    try:
        X = np.full(shape, -1234, np.int16)
        assert ctx.commit(srs, to_device(X), T.TC_I16) == ec.g1_to_bytes(ec.mul(-1234 % R, ec.G1))
        rng = np.random.default_rng(26)
        X[4096:, :] = np.clip(np.rint(rng.standard_normal((4096, 8192)) * 3000.0), -32767, 32767).astype(np.int16)
        assert ctx.commit(srs, to_device(X), T.TC_I16) == ec.g1_to_bytes(cbind.commit(pp, X, nthreads=16))
    finally:
        srs.close()


@pytest.mark.parametrize("shape", [(4096, 4096), (4096, 8192)])
def test_two_level_sort_at_its_limits(T, ctx, shape):
    """Commitments of 2^24 and 2^25 int16 terms, the largest problems that the sort in two levels takes with seven and
    with six lower key bits beside the index of a term: a constant tensor (every entry in one bucket: a bin of thousands
    of tiles, ranks up to the tile's size), a tensor with two non-zero entries, the first and the last (the top bit of
    the index field), and -- at 2^24 -- values on both sides of every kind of bin and key boundary next to a Gaussian
    half, against the oracle's closed form."""
    pp = pps(shape)
    n = tc.prod(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    try:
        X = np.full(shape, 257, np.int16)
        assert ctx.commit(srs, to_device(X), T.TC_I16) == ec.g1_to_bytes(ec.mul(257, ec.G1))
        X[:] = 0
        X.reshape(-1)[0], X.reshape(-1)[-1] = -32768, 129
        want = (-32768 * pp.lagrange_scalar(tc.multi_index(0, shape)) + 129 * pp.lagrange_scalar(tc.multi_index(n - 1, shape))) % R
        assert ctx.commit(srs, to_device(X), T.TC_I16) == ec.g1_to_bytes(cbind.g1_mul(want, ec.G1))
        if n == 1 << 24:
            rng = np.random.default_rng(24)
            X = np.clip(np.rint(rng.standard_normal(shape) * 6300.0), -32767, 32767).astype(np.int16)
            edges = np.array([1, -1, 64, 65, -64, -65, 128, 129, -128, -129, 256, 257, 16384, 16385, -16384, -16385,
                              32767, -32767, -32768, 0, 32640, 32641, -32640, -32641], np.int16)
            X[: shape[0] // 2, :] = np.resize(edges, (shape[0] // 2, shape[1]))
            assert ctx.commit(srs, to_device(X), T.TC_I16) == ec.g1_to_bytes(cbind.commit(pp, X, nthreads=16))
    finally:
        srs.close()


@pytest.mark.parametrize("table", [False, True])
@pytest.mark.parametrize("shape", [(64, 512), (5, 37, 100), (300, 64)])
def test_open_by_rows_matches_oracle(T, ctx, shape, table):
    """Openings of tensors large enough for the row-wise route (two 9-bit digits per entry for the
    leading axes) against the oracle's closed form; int16 incl. extreme differences, and int8; without and with
    the opening table (row commitments + one short problem against U; its entries checked from the definition)."""
    pp = pps(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX | (T.TC_SRS_OPEN_TABLE if table else 0))
    try:
        if table:
            data = srs.export()
            n_suffix = sum(tc.prod(shape[a:]) for a in range(len(shape)))
            inner = tc.prod(shape[1:])
            assert len(data) == 56 + 96 * (n_suffix + tc.prod(shape))
            for kappa, t in ((0, 0), (shape[0] - 1, inner - 1), (shape[0] // 2, inner // 3)):
                g = sum(pp.ell[0][k] * ec.fr_inv(k - kappa) for k in range(shape[0]) if k != kappa) % R
                want = cbind.g1_mul(g * pp.lagrange_scalar(tc.multi_index(t, shape[1:]), 1) % R, ec.G1)
                off = 56 + 96 * (n_suffix + kappa * inner + t)
                assert data[off : off + 96] == ec.g1_to_bytes(want)
        X16 = tc_inputs.int16_uniform(shape, 3, -32768, 32767)
        flat = X16.reshape(shape[0], -1)
        flat[0, 0], flat[-1, -1] = -32768, 32767
        flat[1, :] = flat[0, :]
        X8 = tc_inputs.int8_uniform(shape, 4)
        vk = ctx.vk_from_trapdoor(TAU_BYTES)
        for X, dt in ((X16, T.TC_I16), (X8, T.TC_I8)):
            dX = to_device(X)
            C = ctx.commit(srs, dX, dt)
            for kappa in [tuple(0 for _ in shape), tuple(d - 1 for d in shape)] + tc_inputs.opening_positions(shape, 2, 17):
                y, pi = ctx.open(srs, dX, dt, kappa)
                yo, po = tc.open_(pp, X, kappa)
                assert y == ec.fr_to_bytes(yo)
                assert pi == [ec.g1_to_bytes(p) for p in po]
                assert ctx.verify(vk, shape, C, kappa, y, pi)
    finally:
        srs.close()


def test_linearity(T, ctx):
    shape = (9, 21)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    try:
        A = tc_inputs.int8_uniform(shape, 1).astype(np.int16)
        B = tc_inputs.int8_uniform(shape, 2).astype(np.int16)
        a, b = 37, -91
        lhs = ctx.commit(srs, to_device((a * A + b * B).astype(np.int16)), T.TC_I16)
        CA = ec.g1_from_bytes(ctx.commit(srs, to_device(A), T.TC_I16))
        CB = ec.g1_from_bytes(ctx.commit(srs, to_device(B), T.TC_I16))
        assert lhs == ec.g1_to_bytes(ec.add(ec.mul(a % R, CA), ec.mul(b % R, CB)))
    finally:
        srs.close()


def test_encode_matches_oracle_quantisation(T, ctx):
    import torch

    x = tc_inputs.f16_normal((257, 131), 5)
    x.reshape(-1)[:6] = np.array([0.0, -0.0, 65504.0, -65504.0, 6e-8, np.inf], np.float16)
    for inv in (quantize.inv_scale_for(x[np.isfinite(x)]), np.float32(2.0), np.float32(0.0)):
        dst = torch.empty(x.size, dtype=torch.int16, device="cuda")
        ctx.encode_tensor(to_device(x.view(np.int16)), T.TC_F16, x.size, float(inv), dst)
        ctx.sync()
        want = quantize.quantize_f16(np.where(np.isfinite(x), x, np.float16(0)), inv).reshape(-1)
        got = dst.cpu().numpy()
        finite = np.isfinite(x.reshape(-1))
        assert np.array_equal(got[finite], want[finite])
    # buffers that are not 16-byte aligned take the element-wise kernel: same values
    inv = float(quantize.inv_scale_for(x[np.isfinite(x)]))
    src = torch.empty(x.size + 1, dtype=torch.int16, device="cuda")
    src[1:] = to_device(x.view(np.int16)).reshape(-1)
    dst = torch.empty(x.size + 3, dtype=torch.int16, device="cuda")
    ctx.encode_tensor(src[1:], T.TC_F16, x.size, inv, dst[3:])
    ctx.sync()
    want = quantize.quantize_f16(np.where(np.isfinite(x), x, np.float16(0)), np.float32(inv)).reshape(-1)
    finite = np.isfinite(x.reshape(-1))
    assert np.array_equal(dst[3:].cpu().numpy()[finite], want[finite])
    # pass-through copies of integer tensors, ragged lengths
    for n, dt, code in ((1000003, np.int8, T.TC_I8), (77, np.int8, T.TC_I8), (500009, np.int16, T.TC_I16), (5, np.int16, T.TC_I16)):
        v = np.random.default_rng(n).integers(-100, 100, size=n).astype(dt)
        out = torch.empty(n, dtype=torch.int8 if dt == np.int8 else torch.int16, device="cuda")
        ctx.encode_tensor(to_device(v), code, n, 1.0, out)
        ctx.sync()
        assert np.array_equal(out.cpu().numpy(), v)
    half = np.array([0.25, 0.75, 1.25, -0.25, -0.75], np.float16)
    dst = torch.empty(5, dtype=torch.int16, device="cuda")
    ctx.encode_tensor(to_device(half.view(np.int16)), T.TC_F16, 5, 2.0, dst)
    ctx.sync()
    assert dst.cpu().tolist() == [0, 2, 2, 0, -2]


def test_quant_scale_on_device(T, ctx):
    """The per-tensor scale computed by the library (one pass over the fp16 tensor, result left in device memory):
    bit-equal to the oracle's float32(32767) / amax on the single-layer activation, on tensors of the LLaMA2-7B
    forward's two shapes, all zeros, a single outlier, ragged and unaligned buffers, non-finite values left out;
    then the quantisation that reads it from device memory equals the oracle's tensor."""
    import torch

    rng = np.random.default_rng(41)
    cases = [tc_inputs.c2_activation(), tc_inputs.f16_normal((512, 11008), 77), np.zeros((129, 7), np.float16)]
    outlier = (rng.standard_normal(100003) * 0.001).astype(np.float16)
    outlier[99999] = np.float16(12.5)
    cases.append(outlier)
    odd = rng.standard_normal(8 * 256 * 5 + 3).astype(np.float16)
    odd[[5, 6000]] = [np.inf, np.nan]
    cases.append(odd)
    cases.append(np.array([np.nan], np.float16))
    scale = torch.full((4,), -1.0, dtype=torch.float32, device="cuda")
    for x in cases:
        flat = x.reshape(-1)
        finite = flat[np.isfinite(flat)]
        want = quantize.inv_scale_for(finite) if finite.size else np.float32(0)
        for offset in (0, 3):
            buf = torch.zeros(flat.size + 8, dtype=torch.int16, device="cuda")
            buf[offset : offset + flat.size] = to_device(flat.view(np.int16))
            src = buf[offset : offset + flat.size]
            ctx.quant_scale(src, flat.size, scale[1:])
            ctx.sync()
            got = scale[1:2].cpu().numpy()
            assert got.view(np.uint32)[0] == np.float32(want).view(np.uint32), (x.shape, offset, got[0], want)
            dst = torch.empty(flat.size, dtype=torch.int16, device="cuda")
            ctx.encode_tensor_scaled(src, T.TC_F16, flat.size, scale[1:], dst)
            ctx.sync()
            ref = quantize.quantize_f16(np.where(np.isfinite(flat), flat, np.float16(0)), want)
            ok = np.isfinite(flat)
            assert np.array_equal(dst.cpu().numpy()[ok], ref[ok])
    assert scale[0].item() == -1.0 and scale[2].item() == -1.0        # only the one float was written
    # all of them in shared launches (tc_encode_batch_scaled), aligned and not, an empty tensor among them
    flats = [x.reshape(-1) for x in cases] + [np.zeros(0, np.float16)]
    bufs = [torch.zeros(f.size + 8, dtype=torch.int16, device="cuda") for f in flats]
    srcs = []
    for i, (f, b) in enumerate(zip(flats, bufs)):
        off = 3 if i % 2 else 0
        b[off : off + f.size] = to_device(f.view(np.int16))
        srcs.append(b[off : off + f.size])
    dsts = [torch.full((f.size + 1,), 77, dtype=torch.int16, device="cuda") for f in flats]
    scales = torch.full((len(flats) + 2,), -1.0, dtype=torch.float32, device="cuda")
    ctx.encode_batch_scaled(srcs, [f.size for f in flats], scales[1:], [d[1:] if i % 3 == 1 else d for i, d in enumerate(dsts)])
    ctx.sync()
    got = scales.cpu().numpy()
    assert got[0] == -1.0 and got[-1] == -1.0
    for i, f in enumerate(flats):
        finite = f[np.isfinite(f)]
        want = quantize.inv_scale_for(finite) if finite.size else np.float32(0)
        assert got[1 + i : 2 + i].view(np.uint32)[0] == np.float32(want).view(np.uint32), i
        out = dsts[i].cpu().numpy()
        out = out[1:] if i % 3 == 1 else out[:-1]
        ok = np.isfinite(f)
        ref = quantize.quantize_f16(np.where(ok, f, np.float16(0)), want)
        assert np.array_equal(out[ok], ref[ok]), i
        assert dsts[i][0 if i % 3 == 1 else -1].item() == 77           # nothing written outside the tensor


def _check_tree_against_oracle(ctx, tree, otree):
    assert tree.levels == len(otree.levels)
    for L in range(tree.levels):
        grid, n = tree.level_info(L)
        assert grid == otree.levels[L]["grid"] and n == len(otree.levels[L]["C"])
        for i in range(n):
            assert tree.node(L, i) == ec.g1_to_bytes(otree.levels[L]["C"][tc.multi_index(i, grid)])
    assert tree.root == ec.g1_to_bytes(otree.root)


@pytest.mark.parametrize("grid,dtype_name", [((37, 53), "i16"), ((4, 4), "i8"), ((1, 70), "i8"), ((19, 3), "i16")])
def test_entries_tree_small(T, ctx, node_srs, grid, dtype_name):
    node = tc_inputs.NODE_SHAPE
    X = tc_inputs.int16_uniform(grid, 7) if dtype_name == "i16" else tc_inputs.int8_uniform(grid, 7)
    dt = T.TC_I16 if dtype_name == "i16" else T.TC_I8
    dX = to_device(X)
    tree = ctx.terkle_build_entries(node_srs, dX, dt, grid, node)
    otree = terkle.build(pps, tc.as_flat_ints(X), grid, node)
    try:
        _check_tree_against_oracle(ctx, tree, otree)
        vk = ctx.vk_from_trapdoor(TAU_BYTES)
        leaves = tc_inputs.opening_positions(grid, 5, 3) + [tuple(g - 1 for g in grid), (0, 0)]
        proofs = tree.open_batch(leaves)
        paths = [tree.path(l) for l in leaves]
        values = [ec.fr_to_bytes(int(X[l]) % R) for l in leaves]
        for leaf, proof, path in zip(leaves, proofs, paths):
            steps = terkle.open_path(pps, otree, grid, node, leaf)
            assert proof == serialize_steps(steps)
            assert path.n_steps == len(steps)
        assert ctx.verify_paths_batch(vk, paths, [tree.root] * len(leaves), values, proofs) == [True] * len(leaves)
        # the same proofs under public verification (pairing, host only): no trapdoor involved
        pv = T.binding.PairingVerifier(TAU_BYTES, 2)
        assert pv.verify_path(paths[0], tree.root, values[0], proofs[0])
        assert not pv.verify_path(paths[0], tree.root, ec.fr_to_bytes((int(X[leaves[0]]) + 1) % R), proofs[0])
        pv.close()
        # tampering: leaf value, one byte of a proof element, the root
        wrong = [ec.fr_to_bytes((int(X[l]) + 1) % R) for l in leaves]
        assert ctx.verify_paths_batch(vk, paths, [tree.root] * len(leaves), wrong, proofs) == [False] * len(leaves)
        bad = bytearray(proofs[0])
        bad[10] ^= 1
        assert not ctx.verify_path(vk, paths[0], tree.root, values[0], bytes(bad))
        other_root = ec.g1_to_bytes(ec.add(otree.root, ec.G1))
        assert not ctx.verify_path(vk, paths[0], other_root, values[0], proofs[0])
        # flipped entry: the rebuilt root differs and the old proof no longer verifies against it
        X2 = X.copy()
        X2[leaves[0]] ^= 1
        tree2 = ctx.terkle_build_entries(node_srs, to_device(X2), dt, grid, node)
        assert tree2.root != tree.root
        assert not ctx.verify_path(vk, paths[0], tree2.root, values[0], proofs[0])
        tree2.close()
    finally:
        tree.close()


def test_tensors_tree_small(T, ctx, node_srs):
    node = tc_inputs.NODE_SHAPE
    grid = (5, 3)
    shapes = [(2, 3), (4,), (2, 2, 2), (3, 3), (5,), (2, 2), (6, 7), (1,), (3,), (2, 5), (4, 4), (2, 2, 3), (8,), (3, 2), (9,)]
    leaves = [tc_inputs.int16_uniform(s, 50 + i) for i, s in enumerate(shapes)]
    lsrs = [ctx.setup_from_trapdoor(TAU_BYTES, s, T.TC_SRS_SUFFIX) for s in shapes]
    dl = [to_device(x) for x in leaves]
    tree = ctx.terkle_build_tensors(node_srs, lsrs, dl, [T.TC_I16] * len(shapes), grid, node)
    otree = terkle.build(pps, [tc.as_flat_ints(t) for t in leaves], grid, node, kind="tensors", leaf_shapes=shapes)
    try:
        _check_tree_against_oracle(ctx, tree, otree)
        vk = ctx.vk_from_trapdoor(TAU_BYTES)
        for leaf, inner in (((0, 2), (0, 1, 1)), ((4, 2), (8,)), ((2, 0), (5, 6)), ((1, 0), (1, 2))):
            flat = leaf[0] * 3 + leaf[1]
            proof = tree.open(leaf, inner)
            steps = terkle.open_path(pps, otree, grid, node, leaf, inner)
            assert proof == serialize_steps(steps)
            path = tree.path(leaf, inner)
            value = ec.fr_to_bytes(int(leaves[flat][inner]) % R)
            assert ctx.verify_path(vk, path, tree.root, value, proof)
            assert not ctx.verify_path(vk, path, tree.root, ec.fr_to_bytes(5), proof)
    finally:
        tree.close()
        for s in lsrs:
            s.close()


def test_srs_and_tree_files(T, ctx, node_srs):
    """Def. 4.1 Setup publishes pp: an SRS written out and read back commits and opens like the one it came from
    (points equal to the oracle's); the node SRS read back rebuilds its fixed-base tables; a tree built, saved,
    loaded and opened gives the oracle's proofs; damaged files give error codes."""
    B = T.binding
    shape = (37, 53)
    pp = pps(shape)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    data = srs.export()
    assert len(data) == 56 + 96 * (37 * 53 + 53)
    for i in (0, 1, 52, 53, 1000, 37 * 53 - 1):
        point = cbind.g1_mul(pp.lagrange_scalar(tc.multi_index(i, shape)), ec.G1)
        assert data[56 + 96 * i : 56 + 96 * (i + 1)] == ec.g1_to_bytes(point)
    back = ctx.srs_import(data)
    X = tc_inputs.int16_uniform(shape, 12, -32768, 32767)
    dX = to_device(X)
    want = ec.g1_to_bytes(cbind.commit(pp, X))
    assert ctx.commit(srs, dX, T.TC_I16) == want and ctx.commit(back, dX, T.TC_I16) == want
    assert all(back.point(i, a) == srs.point(i, a) for a, idx in ((0, (0, 7, 1960)), (1, (0, 52))) for i in idx)
    kappa = (36, 17)
    yo, po = tc.open_(pp, X, kappa)
    y, pi = ctx.open(back, dX, T.TC_I16, kappa)
    assert y == ec.fr_to_bytes(yo) and pi == [ec.g1_to_bytes(p) for p in po]
    back.close()
    for blob, code in ((data[:-1], B.TC_ERR_ARG), (data[:30], B.TC_ERR_ARG), (b"X" + data[1:], B.TC_ERR_ARG),
                       (data[:12] + (9).to_bytes(4, "little") + data[16:], B.TC_ERR_ARG),
                       (data[:48] + (5).to_bytes(8, "little") + data[56:], B.TC_ERR_ARG),
                       (data[:24] + (9).to_bytes(4, "little") + data[28:], B.TC_ERR_SHAPE),
                       (data[:200] + bytes([data[200] ^ 4]) + data[201:], B.TC_ERR_RANGE)):
        with pytest.raises(T.TcError) as e:
            ctx.srs_import(blob)
        assert e.value.code == code, (e.value.code, code)
    srs.close()
    # the node SRS through a file: the import rebuilds the fixed-base tables that trees use
    node, grid = tc_inputs.NODE_SHAPE, (37, 53)
    node_back = ctx.srs_import(node_srs.export())
    tree = ctx.terkle_build_entries(node_back, dX, T.TC_I16, grid, node)
    otree = terkle.build(pps, tc.as_flat_ints(X), grid, node)
    assert tree.root == ec.g1_to_bytes(otree.root)
    blob = tree.export()
    assert blob[-96:] == ec.g1_to_bytes(otree.root)
    tree.close()
    loaded = ctx.terkle_build_entries(node_srs, dX, T.TC_I16, grid, node, from_file=blob)
    try:
        _check_tree_against_oracle(ctx, loaded, otree)
        for leaf in [(0, 0), (36, 52), (20, 31)]:
            assert loaded.open(leaf) == serialize_steps(terkle.open_path(pps, otree, grid, node, leaf))
        for bad, code in ((blob[:-96], B.TC_ERR_ARG), (blob[:36] + (5).to_bytes(4, "little") + blob[40:], B.TC_ERR_SHAPE),
                          (blob[:80] + bytes([blob[80] ^ 1]) + blob[81:], B.TC_ERR_RANGE)):
            with pytest.raises(T.TcError) as e:
                ctx.terkle_build_entries(node_srs, dX, T.TC_I16, grid, node, from_file=bad)
            assert e.value.code == code, (e.value.code, code)
    finally:
        loaded.close()
        node_back.close()


def test_c1_single_level_tree(T, ctx, c1):
    srs, X, dX = c1
    shape = tc_inputs.C1_SHAPE
    tree = ctx.terkle_build_entries(srs, dX, T.TC_I8, shape, shape)
    try:
        assert tree.levels == 1
        assert tree.root == ec.g1_to_bytes(tc.commit(pps(shape), X))
        vk = ctx.vk_from_trapdoor(TAU_BYTES)
        leaves = tc_inputs.opening_positions(shape, 8, tc_inputs.tensor_seed(0))
        proofs = tree.open_batch(leaves)
        for leaf, proof in zip(leaves, proofs):
            yo, po = tc.open_(pps(shape), X, leaf)
            assert proof == b"".join(ec.g1_to_bytes(p) for p in po) + ec.fr_to_bytes(yo)
        paths = [tree.path(l) for l in leaves]
        vals = [ec.fr_to_bytes(int(X[l]) % R) for l in leaves]
        assert ctx.verify_paths_batch(vk, paths, [tree.root] * 8, vals, proofs) == [True] * 8
    finally:
        tree.close()


def test_c2_activation_commit(T, ctx):
    """Config 2: one 512 x 4096 fp16 activation, quantised on the GPU, committed as one tensor."""
    import torch

    shape = tc_inputs.C2_SHAPE
    x = tc_inputs.c2_activation()
    inv = quantize.inv_scale_for(x)
    q_want = quantize.quantize_f16(x, inv)
    dq = torch.empty(x.size, dtype=torch.int16, device="cuda")
    ctx.encode_tensor(to_device(x.view(np.int16)), T.TC_F16, x.size, float(inv), dq)
    ctx.sync()
    assert np.array_equal(dq.cpu().numpy().reshape(shape), q_want)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, shape, 0)
    try:
        pp = pps(shape)
        got = ctx.commit(srs, dq, T.TC_I16)
        want = cbind.commit(pp, q_want, nthreads=8)
        assert got == ec.g1_to_bytes(want)
        # SRS spot checks at this size
        rng = np.random.default_rng(2)
        for f in [0, tc.prod(shape) - 1] + [int(v) for v in rng.integers(0, tc.prod(shape), 6)]:
            want_pt = cbind.g1_mul(pp.lagrange_scalar(tc.multi_index(f, shape)), ec.G1)
            assert srs.point(f) == ec.g1_to_bytes(want_pt)
    finally:
        srs.close()


def test_c2_tree_every_node_and_paths(T, ctx, node_srs):
    """Config 2, tree form at full size: (4,4) tree over the 2^21 quantised entries, 139 813 nodes.
    The oracle recomputes EVERY node of every level and the root from the payload alone (closed form per node:
    field sum, then one scalar multiplication in the C oracle, on all host cores), its own verifier accepts the
    GPU's membership proofs, and whole proofs equal the oracle's byte for byte."""
    import torch

    watch = Stopwatch("config 2 tree")
    shape, node = tc_inputs.C2_SHAPE, tc_inputs.NODE_SHAPE
    x = tc_inputs.c2_activation()
    q = quantize.quantize_f16(x, quantize.inv_scale_for(x))
    dq = to_device(q)
    tree = ctx.terkle_build_entries(node_srs, dq, T.TC_I16, shape, node)
    try:
        assert tree.levels == 6
        sizes = [131072, 8192, 512, 32, 4, 1]
        assert [tree.level_info(L)[1] for L in range(6)] == sizes
        ppn = pps(node)
        basis = [ppn.lagrange_scalar(tc.multi_index(k, node)) for k in range(16)]       # L_k(tau) of the node shape

        def node_commitment(Z):
            """[sum_k e(Z_k) L_k(tau)] G: Def. 4.1 Com under the known trapdoor, the multiplication in C"""
            s = 0
            for z, l in zip(Z, basis):
                s += int(z) * l
            return cbind.g1_mul(s % R, ec.G1)

        # level 0 from the payload, then every level from the phi values of the one below
        blocks = q.reshape(128, 4, 1024, 4).transpose(0, 2, 1, 3).reshape(-1, 16)
        levels = []
        with oracle_pool() as pool:
            levels.append(list(pool.map(node_commitment, blocks.tolist(), chunksize=512)))
            watch.lap("oracle: %d bottom nodes" % len(levels[0]))
            grid = (128, 1024)
            while len(levels[-1]) > 1:
                below, bgrid = levels[-1], grid
                grid = tuple(-(-g // 4) for g in bgrid)
                phis = [terkle.phi(c) for c in below]
                Zs = []
                for a0 in range(grid[0]):
                    for a1 in range(grid[1]):
                        Zs.append([phis[(4 * a0 + k // 4) * bgrid[1] + 4 * a1 + k % 4]
                                   if 4 * a0 + k // 4 < bgrid[0] and 4 * a1 + k % 4 < bgrid[1] else 0 for k in range(16)])
                levels.append(list(pool.map(node_commitment, Zs, chunksize=64)))
        watch.lap("oracle: levels 1..5 and the root")
        assert [len(l) for l in levels] == sizes
        blob = tree.export()                               # every commitment of the tree in one transfer
        off = 72
        for L, want in enumerate(levels):
            got = blob[off : off + 96 * len(want)]
            off += 96 * len(want)
            if got != b"".join(ec.g1_to_bytes(c) for c in want):
                bad = [i for i, c in enumerate(want) if got[96 * i : 96 * i + 96] != ec.g1_to_bytes(c)]
                raise AssertionError("level %d: %d of %d nodes differ, first %s" % (L, len(bad), len(want), bad[:5]))
        assert off == len(blob) and tree.root == ec.g1_to_bytes(levels[-1][0])
        for L, i in ((0, 0), (0, 131071), (1, 4097), (4, 3)):                # the single-node accessor agrees with the file
            assert tree.node(L, i) == ec.g1_to_bytes(levels[L][i])
        watch.lap("all 139813 nodes equal the oracle's")

        def oracle_node(level, a):
            """commitment of node `a` (multi-index) at `level`, from payload entries only"""
            if level == 0:
                block = q[4 * a[0] : 4 * a[0] + 4, 4 * a[1] : 4 * a[1] + 4]
                return tc.commit(ppn, block)
            Z = [terkle.phi(oracle_node(level - 1, (4 * a[0] + k // 4, 4 * a[1] + k % 4))) for k in range(16)]
            return tc.commit(ppn, Z)

        assert ec.g1_to_bytes(oracle_node(1, (17, 200))) == ec.g1_to_bytes(levels[1][17 * 256 + 200])   # the pooled closed form = tc.commit
        # membership proofs: accepted by the oracle's verifier and by the library, rejected when tampered
        leaves = tc_inputs.opening_positions(shape, 8, tc_inputs.tensor_seed(1))
        proofs = tree.open_batch(leaves)
        vk = ctx.vk_from_trapdoor(TAU_BYTES)
        root = ec.g1_from_bytes(tree.root)
        for leaf, proof in zip(leaves, proofs):
            assert len(proof) == 6 * (2 * 96 + 32) + 5 * 96
            path = tree.path(leaf)
            steps, step_shapes = parse_proof(path, proof)
            assert step_shapes == [node] * 6
            assert terkle.verify_path(pps, root, [node] * 6, int(q[leaf]), steps)
            assert not terkle.verify_path(pps, root, [node] * 6, int(q[leaf]) + 1, steps)
        # two whole proofs byte for byte: the oracle opens the node tensors along the path, Z from its own levels
        for leaf, proof in list(zip(leaves, proofs))[:2]:
            steps, pos, grid_l = [], leaf, shape
            chain = []
            for L in range(6):
                a, k = (pos[0] // 4, pos[1] // 4), (pos[0] % 4, pos[1] % 4)
                chain.append((L, a, k, grid_l))
                pos, grid_l = a, tuple(-(-g // 4) for g in grid_l)
            for L, a, k, bgrid in reversed(chain):
                if L == 0:
                    Z = [int(v) for v in q[4 * a[0] : 4 * a[0] + 4, 4 * a[1] : 4 * a[1] + 4].reshape(-1)]
                    child = None
                else:
                    Z = [terkle.phi(levels[L - 1][(4 * a[0] + j // 4) * bgrid[1] + 4 * a[1] + j % 4])
                         if 4 * a[0] + j // 4 < bgrid[0] and 4 * a[1] + j % 4 < bgrid[1] else 0 for j in range(16)]
                    child = levels[L - 1][(4 * a[0] + k[0]) * bgrid[1] + 4 * a[1] + k[1]]
                y, pi = tc.open_(ppn, Z, k)
                steps.append((k, y, pi, child))
            assert proof == serialize_steps(steps)
        vals = [ec.fr_to_bytes(int(q[l]) % R) for l in leaves]
        assert ctx.verify_paths_batch(vk, [tree.path(l) for l in leaves], [tree.root] * 8, vals, proofs) == [True] * 8
        watch.lap("8 paths verified, 2 proofs equal the oracle's")
        # incremental updates at this size: two entries change (one to an extreme value); the updated tree must
        # equal a fresh build over the changed payload on the whole path, the oracle recomputes the bottom node,
        # and the old proof of that leaf no longer verifies while a new one does
        for leaf, new in ((leaves[0], -32767), (leaves[3], int(q[leaves[3]]) + 1)):
            delta = new - int(q[leaf])
            q[leaf] = new
            dq.copy_(to_device(q))
            tree.update(leaf, delta)
            fresh = ctx.terkle_build_entries(node_srs, dq, T.TC_I16, shape, node)
            try:
                a = leaf
                for level in range(6):
                    grid, _ = tree.level_info(level)
                    a = (a[0] // 4, a[1] // 4)
                    index = a[0] * grid[1] + a[1]
                    assert tree.node(level, index) == fresh.node(level, index), (leaf, level)
                assert tree.root == fresh.root
            finally:
                fresh.close()
            bottom = (leaf[0] // 4, leaf[1] // 4)
            assert tree.node(0, bottom[0] * 1024 + bottom[1]) == ec.g1_to_bytes(oracle_node(0, bottom))
            proof = tree.open(leaf)
            assert ctx.verify_path(vk, tree.path(leaf), tree.root, ec.fr_to_bytes(new % R), proof)
        assert not ctx.verify_path(vk, tree.path(leaves[0]), tree.root, vals[0], proofs[0])
    finally:
        tree.close()


def _oracle_leaf(shape, seed, nthreads):
    """One fp16 N(0,1) tensor of the activation workloads: the oracle's quantisation and closed-form commitment."""
    x = tc_inputs.f16_normal(shape, seed)
    inv = quantize.inv_scale_for(x)
    qv = quantize.quantize_f16(x, inv)
    return x, inv, qv, cbind.commit(pps(shape), qv, nthreads=nthreads)


@pytest.mark.slow
def test_c3_llama7b_forward_leaf_commitments_and_tree(T, ctx, node_srs):
    """Config 3: 32 layers x {512x4096, 512x4096, 512x11008} int16 tensors as whole-tensor leaves,
    (4,4) tree over the (32, 3) grid.  The scale of every tensor is computed on the device and must equal the
    oracle's; every leaf commitment is compared with the oracle's closed form (field sums in C), the upper tree
    with the oracle's recursive build over those commitments; the configuration's 64 openings are made in one
    batch, all of them pass the oracle's verifier, and eight whole proofs equal the oracle's byte for byte."""
    import torch

    watch = Stopwatch("config 3")
    cfg = tc_inputs.LLAMA7B
    shapes3 = tc_inputs.c3_shapes(cfg)
    layers = int(os.environ.get("TC_TEST_C3_LAYERS", cfg["layers"]))
    grid = (layers, 3)
    srs_by_shape = {}
    for s in set(shapes3):
        srs_by_shape[s] = ctx.setup_from_trapdoor(TAU_BYTES, s, T.TC_SRS_SUFFIX | T.TC_SRS_OPEN_TABLE)
        pps(s)                                             # the oracle's parameters, before the pool needs them
    leaves_q, leaves_d, leaf_srs, leaf_shapes = [], [], [], []
    want_commit = []
    scales = torch.empty(layers * 3, dtype=torch.float32, device="cuda")
    specs = [(s, tc_inputs.tensor_seed(2, 0, layer, kind)) for layer in range(layers) for kind, s in enumerate(shapes3)]
    with oracle_pool() as pool:
        for i, (x, inv, qv, want) in enumerate(pool.map(lambda sp: _oracle_leaf(sp[0], sp[1], 2), specs)):
            s = specs[i][0]
            dx = to_device(x.view(np.int16))
            dq = torch.empty(x.size, dtype=torch.int16, device="cuda")
            ctx.quant_scale(dx, x.size, scales[i:])
            ctx.encode_tensor_scaled(dx, T.TC_F16, x.size, scales[i:], dq)
            ctx.sync()
            assert scales[i].item() == float(inv), "scale of tensor %d" % i
            leaves_q.append(qv)
            leaves_d.append(dq)
            leaf_srs.append(srs_by_shape[s])
            leaf_shapes.append(s)
            want_commit.append(want)
    watch.lap("inputs, device scales and oracle commitments of %d tensors" % len(specs))
    for qv, dq in zip(leaves_q[:3], leaves_d[:3]):
        assert np.array_equal(dq.cpu().numpy(), qv.reshape(-1))
    tree = ctx.terkle_build_tensors(node_srs, leaf_srs, leaves_d, [T.TC_I16] * len(leaves_d), grid, tc_inputs.NODE_SHAPE)
    try:
        for i, w in enumerate(want_commit):
            assert tree.node(0, i) == ec.g1_to_bytes(w), "leaf %d" % i
        # upper levels from the oracle's own leaf commitments
        phis = [terkle.phi(w) for w in want_commit]
        otree = terkle.build(pps, phis, grid, tc_inputs.NODE_SHAPE)
        assert tree.levels == len(otree.levels) + 1
        for L in range(1, tree.levels):
            g, n = tree.level_info(L)
            for i in range(n):
                assert tree.node(L, i) == ec.g1_to_bytes(otree.levels[L - 1]["C"][tc.multi_index(i, g)])
        assert tree.root == ec.g1_to_bytes(otree.root)
        watch.lap("tree equals the oracle's")
        # the configuration's 64 random openings down to tensor entries, one batch
        vk = ctx.vk_from_trapdoor(TAU_BYTES)
        rng = np.random.default_rng(tc_inputs.tensor_seed(2) + 999)
        leaf_idx = [(int(rng.integers(0, layers)), int(rng.integers(0, 3))) for _ in range(64)]
        inner_idx = [tuple(int(rng.integers(0, d)) for d in shapes3[l[1]]) for l in leaf_idx]
        proofs = tree.open_batch(leaf_idx, inner_idx)
        paths = [tree.path(l, i) for l, i in zip(leaf_idx, inner_idx)]
        values = [int(leaves_q[l[0] * 3 + l[1]][i]) for l, i in zip(leaf_idx, inner_idx)]
        root_pt = ec.g1_from_bytes(tree.root)

        def oracle_accepts(j):
            steps, step_shapes = parse_proof(paths[j], proofs[j])
            return (terkle.verify_path(pps, root_pt, step_shapes, values[j], steps),
                    terkle.verify_path(pps, root_pt, step_shapes, values[j] + 1, steps))

        with oracle_pool() as pool:
            verdicts = list(pool.map(oracle_accepts, range(64)))
        assert verdicts == [(True, False)] * 64
        watch.lap("64 openings pass the oracle's verifier")
        for j in range(8):                                 # whole proofs: upper steps from the oracle's tree, last step from its Open
            leaf, inner = leaf_idx[j], inner_idx[j]
            flat = leaf[0] * 3 + leaf[1]
            steps = terkle.open_path(pps, otree, grid, tc_inputs.NODE_SHAPE, leaf)
            k, y, pi, _ = steps[-1]
            steps[-1] = (k, y, pi, want_commit[flat])      # the bottom node of the upper tree carries the leaf tensor's commitment
            yo, po = cbind.open_(pps(leaf_shapes[flat]), leaves_q[flat], inner, HOST_THREADS)
            steps.append((inner, yo, po, None))
            assert proofs[j] == serialize_steps(steps), "proof %d" % j
        watch.lap("8 whole proofs equal the oracle's")
        byte_values = [ec.fr_to_bytes(v % R) for v in values]
        assert ctx.verify_paths_batch(vk, paths, [tree.root] * 64, byte_values, proofs) == [True] * 64
    finally:
        tree.close()
        for s in srs_by_shape.values():
            s.close()


@pytest.mark.slow
def test_c4_weight_matrices_streamed(T, ctx, node_srs):
    """Config 4 at its stated size: the weight matrices of all 32 layers at true shapes (Wq/Wk/Wv/Wo 4096x4096,
    W_gate/W_up 4096x11008, W_down 11008x4096, int8 uniform in [-127,127]; 6.48e9 scalars; TC_TEST_C4_LAYERS takes a
    slice): every matrix commitment against the oracle's closed form, then the (4,4) tree over the (layers, 7)
    grid against the oracle's recursive build."""
    import torch

    watch = Stopwatch("config 4")
    layers = int(os.environ.get("TC_TEST_C4_LAYERS", tc_inputs.LLAMA7B["layers"]))
    progress("config 4: %d of 32 layers" % layers)
    shapes7 = tc_inputs.c4_shapes()
    grid = (layers, 7)
    srs_by_shape = {s: ctx.setup_from_trapdoor(TAU_BYTES, s, 0) for s in set(shapes7)}
    for s in set(shapes7):
        pps(s)
    watch.lap("SRS tables")
    leaves_d, leaf_srs, want = [], [], []
    specs = [(s, tc_inputs.tensor_seed(3, 0, layer, kind)) for layer in range(layers) for kind, s in enumerate(shapes7)]

    def oracle_matrix(sp):
        W = tc_inputs.int8_uniform(sp[0], sp[1], -127, 127)
        return W, cbind.commit(pps(sp[0]), W, nthreads=2)

    with oracle_pool() as pool:
        for i, (W, w) in enumerate(pool.map(oracle_matrix, specs)):
            leaves_d.append(to_device(W))
            leaf_srs.append(srs_by_shape[specs[i][0]])
            want.append(w)
            if i % 56 == 55:
                watch.lap("matrices and oracle commitments up to layer %d" % (i // 7))
    tree = ctx.terkle_build_tensors(node_srs, leaf_srs, leaves_d, [T.TC_I8] * len(leaves_d), grid, tc_inputs.NODE_SHAPE)
    try:
        for i, w in enumerate(want):
            assert tree.node(0, i) == ec.g1_to_bytes(w), "matrix %d" % i
        otree = terkle.build(pps, [terkle.phi(w) for w in want], grid, tc_inputs.NODE_SHAPE)
        assert tree.root == ec.g1_to_bytes(otree.root)
        got = ctx.commit_batch(leaf_srs[:7], leaves_d[:7], [T.TC_I8] * 7)
        assert got == [ec.g1_to_bytes(w) for w in want[:7]]
        watch.lap("%d commitments and the tree equal the oracle's" % len(want))
    finally:
        tree.close()
        for s in srs_by_shape.values():
            s.close()


@pytest.mark.slow
def test_c5_batched_requests(T, ctx, node_srs):
    """Config 5 at its stated size on the GPU: 8 requests x 40 layers x {2048x5120 twice, 2048x13824} int16 from fp16
    N(0,1) (1.58e10 scalars), one tree per request over its (40, 3) grid, 128 path openings per request in one
    batch (1024 in all), all verified in one batch on the GPU; roots differ per request.
    The oracle recomputes every leaf commitment (closed form, field sums in C on all host cores), the upper tree and
    the root of every request (TC_TEST_C5_ORACLE_REQUESTS, default all 8, limits that to the first requests; the
    others then get three sampled leaf commitments, one of each shape, picked by seed); for every request the
    tensor-level opening of two paths is recomputed byte for byte and sixteen whole paths go through its verifier.
    TC_TEST_C5_REQUESTS / _LAYERS / _OPENINGS take a slice; the slice is printed."""
    import torch

    watch = Stopwatch("config 5")
    cfg = tc_inputs.LLAMA13B
    requests = int(os.environ.get("TC_TEST_C5_REQUESTS", cfg["batch"]))
    layers = int(os.environ.get("TC_TEST_C5_LAYERS", cfg["layers"]))
    openings = int(os.environ.get("TC_TEST_C5_OPENINGS", "128"))
    oracle_requests = int(os.environ.get("TC_TEST_C5_ORACLE_REQUESTS", cfg["batch"]))
    progress("config 5: %d of 8 requests x %d of 40 layers, %d openings per request, oracle rebuilds %d request(s) in full"
             % (requests, layers, openings, min(oracle_requests, requests)))
    shapes3 = tc_inputs.c3_shapes(cfg)
    grid = (layers, 3)
    srs_by_shape = {s: ctx.setup_from_trapdoor(TAU_BYTES, s, T.TC_SRS_SUFFIX | T.TC_SRS_OPEN_TABLE) for s in set(shapes3)}
    for s in set(shapes3):
        pps(s)
    watch.lap("SRS tables")
    vk = ctx.vk_from_trapdoor(TAU_BYTES)
    roots, trees, keep = [], [], []
    paths, proofs, values, proof_roots = [], [], [], []

    def quantised(sp):
        x = tc_inputs.f16_normal(sp[0], sp[1])
        inv = quantize.inv_scale_for(x)
        return x, inv, quantize.quantize_f16(x, inv)

    try:
        for req in range(requests):
            full = req < oracle_requests
            specs = [(s, tc_inputs.tensor_seed(4, req, layer, kind)) for layer in range(layers) for kind, s in enumerate(shapes3)]
            rng = np.random.default_rng(tc_inputs.tensor_seed(4, req) + 555)
            sampled = set(range(len(specs))) if full else {3 * int(rng.integers(0, layers)) + kind for kind in range(3)}
            leaves_q, leaves_d, leaf_srs, want = [], [], [], {}
            scales = torch.empty(len(specs), dtype=torch.float32, device="cuda")
            with oracle_pool() as pool:
                pending = {}
                for i, (x, inv, qv) in enumerate(pool.map(quantised, specs)):
                    dx = to_device(x.view(np.int16))
                    dq = torch.empty(x.size, dtype=torch.int16, device="cuda")
                    ctx.quant_scale(dx, x.size, scales[i:])
                    ctx.encode_tensor_scaled(dx, T.TC_F16, x.size, scales[i:], dq)
                    ctx.sync()
                    assert scales[i].item() == float(inv), "scale of tensor %d of request %d" % (i, req)
                    if i in sampled:
                        assert np.array_equal(dq.cpu().numpy(), qv.reshape(-1)), "quantised tensor %d of request %d" % (i, req)
                        pending[i] = pool.submit(cbind.commit, pps(specs[i][0]), qv, 2)
                    leaves_q.append(qv)
                    leaves_d.append(dq)
                    leaf_srs.append(srs_by_shape[specs[i][0]])
                for i, fut in pending.items():
                    want[i] = fut.result()
            watch.lap("request %d: inputs quantised on both sides, %d oracle commitments" % (req, len(want)))
            tree = ctx.terkle_build_tensors(node_srs, leaf_srs, leaves_d, [T.TC_I16] * len(leaves_d), grid, tc_inputs.NODE_SHAPE)
            trees.append(tree)
            keep.append(leaves_d)
            for i, w in want.items():
                assert tree.node(0, i) == ec.g1_to_bytes(w), "leaf %d of request %d" % (i, req)
            if full:
                otree = terkle.build(pps, [terkle.phi(want[i]) for i in range(len(specs))], grid, tc_inputs.NODE_SHAPE)
                assert tree.root == ec.g1_to_bytes(otree.root)
            roots.append(tree.root)
            rng = np.random.default_rng(tc_inputs.tensor_seed(4, req) + 999)
            leaf_idx, inner_idx = [], []
            for _ in range(openings):
                leaf = (int(rng.integers(0, layers)), int(rng.integers(0, 3)))
                leaf_idx.append(leaf)
                inner_idx.append(tuple(int(rng.integers(0, d)) for d in shapes3[leaf[1]]))
            got = tree.open_batch(leaf_idx, inner_idx)
            watch.lap("request %d: tree built, %d openings made" % (req, openings))
            root_pt = ec.g1_from_bytes(tree.root)
            req_paths = [tree.path(l, i) for l, i in zip(leaf_idx, inner_idx)]
            req_values = [int(leaves_q[l[0] * 3 + l[1]][i]) for l, i in zip(leaf_idx, inner_idx)]

            def oracle_check(j):
                leaf, inner, proof = leaf_idx[j], inner_idx[j], got[j]
                flat = leaf[0] * 3 + leaf[1]
                if j < 2:      # the tensor-level opening recomputed by the oracle
                    yo, po = cbind.open_(pps(shapes3[leaf[1]]), leaves_q[flat], inner, 4)
                    tail = b"".join(ec.g1_to_bytes(p) for p in po) + ec.fr_to_bytes(yo)
                    return proof[-len(tail):] == tail
                steps, step_shapes = parse_proof(req_paths[j], proof)      # the whole path through the oracle's verifier
                return (terkle.verify_path(pps, root_pt, step_shapes, req_values[j], steps)
                        and not terkle.verify_path(pps, root_pt, step_shapes, req_values[j] + 1, steps))

            with oracle_pool() as pool:
                assert all(pool.map(oracle_check, range(min(openings, 18))))
            paths += req_paths
            proofs += got
            values += [ec.fr_to_bytes(v % R) for v in req_values]
            proof_roots += [tree.root] * openings
            watch.lap("request %d: oracle checked %d openings" % (req, min(openings, 18)))
        assert len(set(roots)) == requests
        assert ctx.verify_paths_batch(vk, paths, proof_roots, values, proofs) == [True] * len(paths)
        watch.lap("%d paths verified in one batch on the GPU" % len(paths))
        if requests > 1:   # a proof of request 0 does not verify against the root of request 1
            assert not ctx.verify_path(vk, paths[0], roots[1], values[0], proofs[0])
    finally:
        for t in trees:
            t.close()
        for s in srs_by_shape.values():
            s.close()


def _coeff_list(t):
    raw = t.cpu().numpy().tobytes()
    return [int.from_bytes(raw[32 * i : 32 * (i + 1)], "little") for i in range(len(raw) // 32)]


def test_coefficient_route(T, ctx):
    """Interpolation to monomial coefficients and Algorithm 1 on the GPU against the oracle's literal route
    (Def. 4.1 as printed), over the reshapes of N = 2^12 samples that Fig. 1 sweeps and the C1 shape; then
    commitments and an opening through the monomial SRS against the Lagrange-basis route."""
    import torch

    rng = np.random.default_rng(31)
    for shape in ((64, 64), (16, 16, 16), (8, 8, 8, 8), (4,) * 6, (2,) * 12, (256,), tc_inputs.C1_SHAPE, (300, 7)):
        n = int(np.prod(shape))
        X = rng.integers(-32768, 32768, size=shape).astype(np.int16)
        coeffs = torch.empty(32 * n, dtype=torch.uint8, device="cuda")
        ctx.interpolate(shape, to_device(X), T.TC_I16, coeffs)
        want = tc.interpolate(X, shape)
        assert _coeff_list(coeffs) == want, shape
        for form in (T.TC_INTERP_NEWTON, T.TC_INTERP_GREGORY, T.TC_INTERP_BARYCENTRIC):     # the three forms of App. C
            by_form = torch.empty_like(coeffs)
            ctx.interpolate_form(shape, to_device(X), T.TC_I16, form, by_form)
            assert _coeff_list(by_form) == want, (shape, form)
        axis = len(shape) - 1 if len(shape) > 1 else 0
        kap = int(rng.integers(0, shape[axis]))
        q = torch.empty_like(coeffs)
        r = torch.empty_like(coeffs)
        ctx.divide_by_linear(shape, coeffs, axis, kap, q, r)
        qo, ro = tc.divide_by_linear(want, shape, axis, kap + 1)
        assert _coeff_list(q) == qo and _coeff_list(r) == ro, shape
    # the longest line of the sweep, N = 2^12 in one axis: the polynomial must reproduce the samples on the grid
    X = rng.integers(-128, 128, size=(4096,)).astype(np.int8)
    coeffs = torch.empty(32 * 4096, dtype=torch.uint8, device="cuda")
    ctx.interpolate((4096,), to_device(X), T.TC_I8, coeffs)
    a = _coeff_list(coeffs)
    for k in (0, 1, 2, 777, 2048, 4094, 4095):
        acc = 0
        for c in reversed(a):
            acc = (acc * (k + 1) + c) % R
        assert acc == int(X[k]) % R, k
    for form in (T.TC_INTERP_GREGORY, T.TC_INTERP_BARYCENTRIC):
        by_form = torch.empty_like(coeffs)
        ctx.interpolate_form((4096,), to_device(X), T.TC_I8, form, by_form)
        assert _coeff_list(by_form) == a, form
    # commitments and a literal opening at the C1 shape
    shape = tc_inputs.C1_SHAPE
    pp = pps(shape)
    mono = ctx.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_MONOMIAL)
    lag = ctx.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    try:
        X = tc_inputs.c1_tensor()
        dX = to_device(X)
        n = int(np.prod(shape))
        coeffs = torch.empty(32 * n, dtype=torch.uint8, device="cuda")
        ctx.interpolate(shape, dX, T.TC_I8, coeffs)
        C = ctx.commit(mono, coeffs, T.TC_FR)
        assert C == ctx.commit(lag, dX, T.TC_I8) == ec.g1_to_bytes(tc.commit(pp, X))
        kappa = (1, 7, 12)
        rem, proof = coeffs, []
        for axis in range(3):
            q, r = torch.empty_like(coeffs), torch.empty_like(coeffs)
            ctx.divide_by_linear(shape, rem, axis, kappa[axis], q, r)
            proof.append(ctx.commit(mono, q, T.TC_FR))
            rem = r
        y, pi = ctx.open(lag, dX, T.TC_I8, kappa)
        assert proof == pi
        assert _coeff_list(rem)[0] == ec.fr_from_bytes(y) == int(X[kappa]) % R and not any(_coeff_list(rem)[1:])
    finally:
        mono.close()
        lag.close()


def test_coefficient_route_at_the_size_the_bench_times(T, ctx):
    """Interpolation of the whole 512 x 4096 activation, the size bench.py times: the three forms of App. C return
    the same coefficient array, and the polynomial reproduces sampled entries of the tensor (what can be computed
    one by one on the CPU at this size)."""
    import torch

    shape = tc_inputs.C2_SHAPE
    x = tc_inputs.c2_activation()
    q = np.clip(np.rint(x.astype(np.float32) * 1000.0), -32767, 32767).astype(np.int16)
    dq = to_device(q)
    n = q.size
    newton = torch.empty(32 * n, dtype=torch.uint8, device="cuda")
    ctx.interpolate(shape, dq, T.TC_I16, newton)
    for form in (T.TC_INTERP_GREGORY, T.TC_INTERP_BARYCENTRIC):
        other = torch.empty_like(newton)
        ctx.interpolate_form(shape, dq, T.TC_I16, form, other)
        assert torch.equal(other, newton), form
        del other
    raw = newton.cpu().numpy().reshape(shape[0], shape[1], 32)
    for (i, j) in ((0, 0), (511, 4095), (137, 2049)):
        # f(i + 1, j + 1) by Horner: along axis 1 for every row of coefficients, then along axis 0
        acc = 0
        for a in range(shape[0] - 1, -1, -1):
            row = 0
            for b in range(shape[1] - 1, -1, -1):
                row = (row * (j + 1) + int.from_bytes(raw[a, b].tobytes(), "little")) % R
            acc = (acc * (i + 1) + row) % R
        assert acc == int(q[i, j]) % R, (i, j)


@pytest.mark.parametrize("node,grid", [((8, 8), (64, 64)), ((4, 4, 4), (16, 16, 16)), ((64,), (4096,)), ((8, 8), (70, 9))])
def test_arity_64_trees(T, ctx, node, grid):
    """The tree shapes of the paper's tree-scaling comparison (Fig. 4, B = 64): Terkle nodes (8,8) and (4,4,4),
    and the Verkle tree as the order-1 node shape (64,), over 64^2 leaves (and a ragged grid): every node, paths,
    batch verification, and an incremental update against the oracle's rebuild."""
    X = tc_inputs.int16_uniform(grid, 11)
    dX = to_device(X)
    srs = ctx.setup_from_trapdoor(TAU_BYTES, node, T.TC_SRS_SUFFIX | T.TC_SRS_FIXED_BASE)
    tree = ctx.terkle_build_entries(srs, dX, T.TC_I16, grid, node)
    try:
        otree = terkle.build(pps, tc.as_flat_ints(X), grid, node)
        _check_tree_against_oracle(ctx, tree, otree)
        vk = ctx.vk_from_trapdoor(TAU_BYTES)
        leaves = tc_inputs.opening_positions(grid, 3, 5) + [tuple(g - 1 for g in grid)]
        proofs = tree.open_batch(leaves)
        for leaf, proof in zip(leaves, proofs):
            assert proof == serialize_steps(terkle.open_path(pps, otree, grid, node, leaf))
        values = [ec.fr_to_bytes(int(X[l]) % R) for l in leaves]
        paths = [tree.path(l) for l in leaves]
        assert ctx.verify_paths_batch(vk, paths, [tree.root] * len(leaves), values, proofs) == [True] * len(leaves)
        pv = T.PairingVerifier(TAU_BYTES, len(node))
        assert pv.verify_path(paths[0], tree.root, values[0], proofs[0])
        pv.close()
        # one entry changes
        leaf = leaves[1]
        new = -int(X[leaf]) - 3
        delta = new - int(X[leaf])
        X[leaf] = new
        dX.copy_(to_device(X))
        tree.update(leaf, delta)
        otree = terkle.build(pps, tc.as_flat_ints(X), grid, node)
        _check_tree_against_oracle(ctx, tree, otree)
        proof = tree.open(leaf)
        assert proof == serialize_steps(terkle.open_path(pps, otree, grid, node, leaf))
        assert ctx.verify_path(vk, tree.path(leaf), tree.root, ec.fr_to_bytes(new % R), proof)
    finally:
        tree.close()
        srs.close()


def test_verification_in_chunks(T, ctx, node_srs):
    """More steps than one pass of the verifier holds (4096): 1400 paths of 3 steps through a (64, 64) entries tree,
    a few of them with a wrong value or a damaged proof; the verdicts must come out per path, in order."""
    grid, node = (64, 64), tc_inputs.NODE_SHAPE
    X = tc_inputs.int16_uniform(grid, 21)
    tree = ctx.terkle_build_entries(node_srs, to_device(X), T.TC_I16, grid, node)
    try:
        otree = terkle.build(pps, tc.as_flat_ints(X), grid, node)
        assert tree.root == ec.g1_to_bytes(otree.root)
        rng = np.random.default_rng(22)
        leaves = [(int(a), int(b)) for a, b in rng.integers(0, 64, size=(1400, 2))]
        proofs = tree.open_batch(leaves)
        for i in (0, 699, 1399):
            assert proofs[i] == serialize_steps(terkle.open_path(pps, otree, grid, node, leaves[i]))
        paths = [tree.path(l) for l in leaves]
        values = [ec.fr_to_bytes(int(X[l]) % R) for l in leaves]
        want = [True] * len(leaves)
        for i in (3, 1365, 1366, 1399):                     # the last ones fall into the second pass
            values[i] = ec.fr_to_bytes((int(X[leaves[i]]) + 1) % R)
            want[i] = False
        damaged = bytearray(proofs[1370])
        damaged[100] ^= 1
        proofs[1370] = bytes(damaged)
        want[1370] = False
        vk = ctx.vk_from_trapdoor(TAU_BYTES)
        assert ctx.verify_paths_batch(vk, paths, [tree.root] * len(leaves), values, proofs) == want
    finally:
        tree.close()
