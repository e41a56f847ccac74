"""CPU tests of the library's host logic and C ABI (no GPU needed).

Two things are exercised here:
  * the product library libtc.so loads and exports every symbol include/tc.h declares
    (no compute call is made without a GPU);
  * a host-emulation build of the same sources (g++ -DTC_HOST_EMU: every kernel functor
    is run lane by lane on the CPU) is driven through the same C ABI and compared with
    the oracle byte for byte.  This checks launch planning, sorting passes, level loops,
    proof assembly and the error paths; the HIP code path itself is checked by the
    `-m gpu` tests.  The emulation build is never loaded by the package."""
import ctypes
import os
import re
import sys

import numpy as np
import pytest

import tc_inputs
from oracle import bls12_381 as ec
from oracle import tc, terkle
from oracle.bls12_381 import R

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import __graft_entry__ as entry  # noqa: E402
import paper_2602_12630_amd as T  # noqa: E402
from gpu_util import TAU_BYTES, check_field_arithmetic, check_one_point_throughout, check_repeated_points, fr_bytes_array, pps, serialize_steps  # noqa: E402

EMU = os.path.join(ROOT, "tests", "hostmath", "libtc_hostemu.so")


def declared_symbols():
    with open(os.path.join(ROOT, "include", "tc.h")) as f:
        text = f.read()
    return sorted(set(re.findall(r"\b(tc_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported_by_the_product_library():
    if not os.path.exists(T.library_path()):
        entry.build_hip()
    lib = T.load_library()
    names = declared_symbols()
    assert len(names) >= 25
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(lib._tc_signatures), "binding and header disagree"


def test_product_library_fails_loudly_without_a_gpu():
    import torch

    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(T.TcError) as e:
        T.Context(0)
    assert e.value.code == T.binding.TC_ERR_HIP


@pytest.fixture(scope="module")
def emu():
    src = [os.path.join(ROOT, "paper_2602_12630_amd", "csrc", f) for f in os.listdir(os.path.join(ROOT, "paper_2602_12630_amd", "csrc"))]
    if not os.path.exists(EMU) or os.path.getmtime(EMU) < max(os.path.getmtime(f) for f in src + [os.path.join(ROOT, "include", "tc.h")]):
        entry.build_host_emulation(EMU)
    lib = T.load_library(EMU)
    ctx = T.Context(0, None, lib)
    yield ctx
    ctx.close()


@pytest.fixture(scope="module")
def node_srs(emu):
    s = emu.setup_from_trapdoor(TAU_BYTES, (2, 2), T.TC_SRS_SUFFIX | T.TC_SRS_FIXED_BASE)
    yield s
    s.close()


def test_emulated_commit_open_verify(emu):
    shape = (3, 4, 2)
    pp = pps(shape)
    srs = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    S = pp.srs_lagrange(0)
    assert all(srs.point(i) == ec.g1_to_bytes(S[i]) for i in range(24))
    assert all(srs.point(i, 2) == ec.g1_to_bytes(pp.srs_lagrange(2)[i]) for i in range(2))
    X16 = tc_inputs.int16_uniform(shape, 5, -32768, 32767)
    X8 = tc_inputs.int8_uniform(shape, 5)
    assert emu.commit(srs, X16, T.TC_I16) == ec.g1_to_bytes(tc.commit(pp, X16))
    assert emu.commit(srs, X8, T.TC_I8) == ec.g1_to_bytes(tc.commit(pp, X8))
    fr = fr_bytes_array([int(v) for v in X16.reshape(-1)])
    assert emu.commit(srs, fr, T.TC_FR) == ec.g1_to_bytes(tc.commit(pp, X16))
    assert emu.commit(srs, np.zeros(shape, np.int16), T.TC_I16) == bytes(96)
    assert emu.commit(srs, np.full(shape, -7, np.int16), T.TC_I16) == ec.g1_to_bytes(ec.mul(-7 % R, ec.G1))
    C = emu.commit(srs, X16, T.TC_I16)
    vk = emu.vk_from_trapdoor(TAU_BYTES)
    for kappa in [(1, 2, 1), (0, 0, 0), (2, 3, 1)]:
        y, pi = emu.open(srs, X16, T.TC_I16, kappa)
        yo, po = tc.open_(pp, X16, kappa)
        assert y == ec.fr_to_bytes(yo) and pi == [ec.g1_to_bytes(p) for p in po]
        assert emu.verify(vk, shape, C, kappa, y, pi)
        assert not emu.verify(vk, shape, C, kappa, ec.fr_to_bytes((yo + 1) % R), pi)
    both = emu.commit_batch([srs, srs], [X16, X8], [T.TC_I16, T.TC_I8])
    assert both == [ec.g1_to_bytes(tc.commit(pp, X16)), ec.g1_to_bytes(tc.commit(pp, X8))]
    # nine int16 tensors in one batch: launches with that many 32768-bucket windows take the packed row / column sums
    rng = np.random.default_rng(77)
    many = [rng.integers(-32767, 32768, size=shape).astype(np.int16) for _ in range(9)]
    many[3][...] = 0
    many[5].reshape(-1)[:] = 32767
    many[6].reshape(-1)[:] = -32767
    got = emu.commit_batch([srs] * 9, many, [T.TC_I16] * 9)
    assert got == [ec.g1_to_bytes(tc.commit(pp, X)) for X in many]
    srs.close()


@pytest.mark.parametrize("shape", [(48, 131), (24, 85)])
def test_emulated_int16_commits_over_several_tiles(emu, shape):
    """Tensors of a few thousand 16-bit terms span several ragged tiles of the count / scatter kernels, which read
    sixteen bytes per lane where a tile is aligned and single values elsewhere.  Commitments alone, as a batch, and
    from a buffer at an odd offset, against the oracle's closed form; extreme and repeated values, a tensor of zeros.
    In this build the two sizes take the two word layouts of the sort in two levels (six and seven lower key bits),
    with tiles of 64 entries: many tiles per bin, the heavily loaded bucket several tiles of its own."""
    pp = pps(shape)
    srs = emu.setup_from_trapdoor(TAU_BYTES, shape, 0)
    rng = np.random.default_rng(9)
    gauss = np.clip(np.rint(rng.standard_normal(shape) * 7000), -32767, 32767).astype(np.int16)
    edge = rng.integers(-32768, 32768, size=shape).astype(np.int16)
    edge.reshape(-1)[::7] = 0
    edge.reshape(-1)[1::97] = -32768
    edge.reshape(-1)[2::89] = 32767
    edge.reshape(-1)[3::5] = 255                       # one heavily loaded bucket
    edge.reshape(-1)[4::11] = -256
    zeros = np.zeros(shape, np.int16)
    for X in (gauss, edge):
        assert emu.commit(srs, X, T.TC_I16) == ec.g1_to_bytes(tc.commit(pp, X))
    got = emu.commit_batch([srs] * 3, [gauss, zeros, edge], [T.TC_I16] * 3)
    assert got == [ec.g1_to_bytes(tc.commit(pp, X)) for X in (gauss, zeros, edge)]
    for off in (1, 3, 8):
        buf = np.zeros(gauss.size + 16, np.int16)
        buf[off : off + gauss.size] = gauss.reshape(-1)
        assert emu.commit(srs, buf[off : off + gauss.size], T.TC_I16) == ec.g1_to_bytes(tc.commit(pp, gauss)), off
    srs.close()


def test_emulated_open_by_rows(emu):
    """Openings along a leading axis of a larger tensor take the row-wise route (17-bit numerators as two
    9-bit digits per entry); same bytes as the oracle's closed form."""
    shape = (8, 2048)
    pp = pps(shape)
    srs = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    try:
        X16 = tc_inputs.int16_uniform(shape, 3, -32768, 32767)
        X16[0, 0], X16[7, 2047], X16[3, 77] = -32768, 32767, -32768
        X16[4, :] = X16[3, :]                                    # a row equal to the opened row: zero numerators
        X8 = tc_inputs.int8_uniform(shape, 4)
        for X, dt in ((X16, T.TC_I16), (X8, T.TC_I8)):
            for kappa in [(3, 77), (0, 0), (7, 2047)]:
                y, pi = emu.open(srs, X, dt, kappa)
                yo, po = tc.open_(pp, X, kappa)
                assert y == ec.fr_to_bytes(yo)
                assert pi == [ec.g1_to_bytes(p) for p in po]
    finally:
        srs.close()
    # many rows: the bucket reduction of the row problems switches to the 16 x 16 form
    shape = (260, 64)
    pp = pps(shape)
    srs = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    try:
        X = tc_inputs.int16_uniform(shape, 6, -32768, 32767)
        for kappa in [(0, 63), (259, 0), (100, 31)]:
            y, pi = emu.open(srs, X, T.TC_I16, kappa)
            yo, po = tc.open_(pp, X, kappa)
            assert y == ec.fr_to_bytes(yo) and pi == [ec.g1_to_bytes(p) for p in po]
    finally:
        srs.close()


def test_emulated_entries_tree(emu, node_srs):
    node, grid = (2, 2), (5, 7)
    X = tc_inputs.int16_uniform(grid, 7)
    tree = emu.terkle_build_entries(node_srs, X, T.TC_I16, grid, node)
    ot = terkle.build(pps, tc.as_flat_ints(X), grid, node)
    assert tree.levels == len(ot.levels) == 3
    for L in range(tree.levels):
        g, n = tree.level_info(L)
        assert g == ot.levels[L]["grid"]
        for i in range(n):
            assert tree.node(L, i) == ec.g1_to_bytes(ot.levels[L]["C"][tc.multi_index(i, g)])
    assert tree.root == ec.g1_to_bytes(ot.root)
    vk = emu.vk_from_trapdoor(TAU_BYTES)
    leaves = [(0, 0), (4, 6), (2, 3)]
    proofs = tree.open_batch(leaves)
    for leaf, proof in zip(leaves, proofs):
        assert proof == serialize_steps(terkle.open_path(pps, ot, grid, node, leaf))
        path = tree.path(leaf)
        val = ec.fr_to_bytes(int(X[leaf]) % R)
        assert emu.verify_path(vk, path, tree.root, val, proof)
        assert not emu.verify_path(vk, path, tree.root, ec.fr_to_bytes((int(X[leaf]) + 1) % R), proof)
        bad = bytearray(proof)
        bad[100] ^= 1
        assert not emu.verify_path(vk, path, tree.root, val, bytes(bad))
        assert not emu.verify_path(vk, path, tree.root, val, proof[:-1])
    tree.close()


def test_emulated_tensors_tree_and_single_node_tree(emu, node_srs):
    node, grid = (2, 2), (3, 2)
    shapes = [(2, 3), (4,), (2, 2, 2), (3, 3), (5,), (2, 2)]
    leaves = [tc_inputs.int16_uniform(s, 50 + i) for i, s in enumerate(shapes)]
    lsrs = [emu.setup_from_trapdoor(TAU_BYTES, s, T.TC_SRS_SUFFIX) for s in shapes]
    tree = emu.terkle_build_tensors(node_srs, lsrs, leaves, [T.TC_I16] * 6, grid, node)
    ot = terkle.build(pps, [tc.as_flat_ints(t) for t in leaves], grid, node, kind="tensors", leaf_shapes=shapes)
    assert tree.root == ec.g1_to_bytes(ot.root) and tree.levels == 3
    proof = tree.open((1, 0), (1, 0, 1))
    assert proof == serialize_steps(terkle.open_path(pps, ot, grid, node, (1, 0), (1, 0, 1)))
    vk = emu.vk_from_trapdoor(TAU_BYTES)
    assert emu.verify_path(vk, tree.path((1, 0), (1, 0, 1)), tree.root, ec.fr_to_bytes(int(leaves[2][1, 0, 1]) % R), proof)
    tree.close()
    # a node shape without fixed-base tables: every node goes through the general engine
    shape = (2, 4, 4)
    X = tc_inputs.int8_uniform(shape, 9)
    big = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    t1 = emu.terkle_build_entries(big, X, T.TC_I8, shape, shape)
    assert t1.levels == 1 and t1.root == ec.g1_to_bytes(tc.commit(pps(shape), X))
    yo, po = tc.open_(pps(shape), X, (1, 2, 3))
    assert t1.open((1, 2, 3)) == b"".join(ec.g1_to_bytes(p) for p in po) + ec.fr_to_bytes(yo)
    t1.close()
    for s in lsrs + [big]:
        s.close()


def test_error_paths(emu, node_srs):
    B = T.binding
    lib = emu.lib
    h = ctypes.c_void_p()
    assert lib.tc_ctx_create(None, 0, None) == B.TC_ERR_ARG
    shape2 = (ctypes.c_uint32 * 4)(3, 4, 1, 1)
    # setup: bad order, zero extent, trapdoor on the grid / zero / non-canonical
    assert lib.tc_setup_from_trapdoor(emu.handle, TAU_BYTES, 5, shape2, 0, ctypes.byref(h)) == B.TC_ERR_SHAPE
    assert lib.tc_setup_from_trapdoor(emu.handle, TAU_BYTES, 2, (ctypes.c_uint32 * 4)(3, 0), 0, ctypes.byref(h)) == B.TC_ERR_SHAPE
    on_grid = (3).to_bytes(32, "little") + TAU_BYTES[32:]
    assert lib.tc_setup_from_trapdoor(emu.handle, on_grid, 2, shape2, 0, ctypes.byref(h)) == B.TC_ERR_RANGE
    assert lib.tc_setup_from_trapdoor(emu.handle, bytes(32) + TAU_BYTES[32:], 2, shape2, 0, ctypes.byref(h)) == B.TC_ERR_RANGE
    assert lib.tc_setup_from_trapdoor(emu.handle, b"\xff" * 32 + TAU_BYTES[32:], 2, shape2, 0, ctypes.byref(h)) == B.TC_ERR_RANGE
    assert lib.tc_setup_from_trapdoor(emu.handle, TAU_BYTES, 2, (ctypes.c_uint32 * 4)(9, 9), B.TC_SRS_FIXED_BASE, ctypes.byref(h)) == B.TC_ERR_SHAPE
    assert b"fixed-base" in lib.tc_last_error(emu.handle)
    assert lib.tc_setup_from_trapdoor(emu.handle, None, 2, shape2, 0, ctypes.byref(h)) == B.TC_ERR_ARG
    srs = emu.setup_from_trapdoor(TAU_BYTES, (3, 4), 0)               # no suffix tables
    X = tc_inputs.int16_uniform((3, 4), 1)
    out = ctypes.create_string_buffer(96)
    assert lib.tc_commit(emu.handle, srs.handle, None, B.TC_I16, out) == B.TC_ERR_ARG
    assert lib.tc_commit(emu.handle, srs.handle, X.ctypes.data, 9, out) == B.TC_ERR_ARG
    assert lib.tc_commit(emu.handle, srs.handle, X.ctypes.data, B.TC_F16, out) == B.TC_ERR_ARG
    assert lib.tc_commit(emu.handle, None, X.ctypes.data, B.TC_I16, out) == B.TC_ERR_ARG
    with pytest.raises(T.TcError) as e:
        emu.open(srs, X, T.TC_I16, (1, 1))
    assert e.value.code == B.TC_ERR_STATE
    full = emu.setup_from_trapdoor(TAU_BYTES, (3, 4), T.TC_SRS_SUFFIX)
    with pytest.raises(T.TcError) as e:
        emu.open(full, X, T.TC_I16, (3, 0))
    assert e.value.code == B.TC_ERR_RANGE
    with pytest.raises(T.TcError) as e:
        srs.point(12)
    assert e.value.code == B.TC_ERR_RANGE
    with pytest.raises(T.TcError) as e:
        emu.encode_tensor(X, 9, 12, 1.0, X)
    assert e.value.code == B.TC_ERR_ARG
    with pytest.raises(T.TcError) as e:
        emu.encode_tensor(X, T.TC_F16, 12, float("nan"), X)
    assert e.value.code == B.TC_ERR_RANGE
    # tree: node SRS of the wrong shape, bad payload dtype, leaf outside the grid, short proof buffer
    with pytest.raises(T.TcError) as e:
        emu.terkle_build_entries(full, X, T.TC_I16, (3, 4), (2, 2))
    assert e.value.code == B.TC_ERR_SHAPE
    with pytest.raises(T.TcError) as e:
        emu.terkle_build_entries(node_srs, X, T.TC_FR, (3, 4), (2, 2))
    assert e.value.code == B.TC_ERR_ARG
    tree = emu.terkle_build_entries(node_srs, X, T.TC_I16, (3, 4), (2, 2))
    with pytest.raises(T.TcError) as e:
        tree.open((3, 0))
    assert e.value.code == B.TC_ERR_RANGE
    with pytest.raises(T.TcError) as e:
        tree.open_batch([(0, 0)], stride=100)
    assert e.value.code == B.TC_ERR_ARG
    with pytest.raises(T.TcError):
        emu.path_from_grid((3, 4), (2, 2), T.TC_LEAF_ENTRIES, (0, 4))
    # verification: malformed proofs are rejections, not errors
    vk = emu.vk_from_trapdoor(TAU_BYTES)
    path = tree.path((1, 1))
    proof = tree.open((1, 1))
    val = ec.fr_to_bytes(int(X[1, 1]) % R)
    assert emu.verify_path(vk, path, tree.root, val, proof)
    assert not emu.verify_path(vk, path, tree.root, val, proof + b"\0")
    not_on_curve = bytearray(proof)
    not_on_curve[0:96] = (5).to_bytes(48, "little") + (7).to_bytes(48, "little")
    assert not emu.verify_path(vk, path, tree.root, val, bytes(not_on_curve))
    big_y = bytearray(proof)
    big_y[192:224] = b"\xff" * 32
    assert not emu.verify_path(vk, path, tree.root, val, bytes(big_y))
    h2 = ctypes.c_void_p()
    assert lib.tc_vk_from_trapdoor(b"\xff" * 128, 4, ctypes.byref(h2)) == B.TC_ERR_RANGE
    assert lib.tc_vk_from_trapdoor(TAU_BYTES, 0, ctypes.byref(h2)) == B.TC_ERR_ARG
    tree.close()
    srs.close()
    full.close()


def test_path_from_grid_matches_oracle_paths(emu):
    grid, node = (37, 53), (4, 4)
    for leaf in [(0, 0), (36, 52), (17, 5)]:
        p = emu.path_from_grid(grid, node, T.TC_LEAF_ENTRIES, leaf)
        # levels: (10,14) -> (3,4) -> (1,1): three steps, top first
        assert p.n_steps == 3
        pos = leaf
        want = []
        for _ in range(3):
            want.append(tuple(x % d for x, d in zip(pos, node)))
            pos = tuple(x // d for x, d in zip(pos, node))
        got = [tuple(p.kappa[s][j] for j in range(2)) for s in range(3)]
        assert got == want[::-1]


def _fr_array(n):
    return np.zeros(32 * n, dtype=np.uint8)


def _fr_list(buf):
    raw = buf.tobytes()
    return [int.from_bytes(raw[32 * i : 32 * (i + 1)], "little") for i in range(len(raw) // 32)]


def test_emulated_coefficient_route(emu):
    """The literal route of Def. 4.1 through the library: interpolation to monomial coefficients, Algorithm 1 on
    the coefficient array, commitments against the monomial SRS -- each against the oracle's own literal route,
    and the resulting group elements against the Lagrange-basis route."""
    rng = np.random.default_rng(21)
    for shape in ((5,), (3, 4), (2, 3, 2), (1, 4), (2, 2, 2, 2, 2), (7, 1, 3)):
        n = int(np.prod(shape))
        X = rng.integers(-128, 128, size=shape).astype(np.int8)
        coeffs = _fr_array(n)
        emu.interpolate(shape, X, T.TC_I8, coeffs)
        want = tc.interpolate(X, shape)
        assert _fr_list(coeffs) == want, shape
        # the three forms of App. C, each against the oracle's own version of that form
        for form, name in ((T.TC_INTERP_NEWTON, "newton"), (T.TC_INTERP_GREGORY, "gregory"), (T.TC_INTERP_BARYCENTRIC, "barycentric")):
            by_form = _fr_array(n)
            emu.interpolate_form(shape, X, T.TC_I8, form, by_form)
            assert _fr_list(by_form) == tc.interpolate_form(X, shape, name) == want, (shape, name)
        # Algorithm 1 along every axis at some position
        for axis, d in enumerate(shape):
            kap = int(rng.integers(0, d))
            q, r = _fr_array(n), _fr_array(n)
            emu.divide_by_linear(shape, coeffs, axis, kap, q, r)
            qo, ro = tc.divide_by_linear(want, shape, axis, kap + 1)
            assert _fr_list(q) == qo and _fr_list(r) == ro, (shape, axis)
    # int16 and full-width inputs
    X16 = rng.integers(-32768, 32768, size=(4, 3)).astype(np.int16)
    c16 = _fr_array(12)
    emu.interpolate((4, 3), X16, T.TC_I16, c16)
    assert _fr_list(c16) == tc.interpolate(X16, (4, 3))
    big = [int(v) for v in rng.integers(1, 2**62, size=6)]
    big = [(v * v * v) % R for v in big]
    cfr = _fr_array(6)
    emu.interpolate((6,), fr_bytes_array(big), T.TC_FR, cfr)
    assert _fr_list(cfr) == tc.interpolate(big, (6,))
    with pytest.raises(T.TcError):
        emu.interpolate_form((4, 3), X16, T.TC_I16, 3, c16)
    # commitments and an opening through the monomial SRS
    shape = (3, 4)
    pp = pps(shape)
    mono = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_MONOMIAL)
    lag = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    try:
        srs_mono = pp.srs_monomial()
        for k in (0, 1, 5, 11):
            assert mono.point(k) == ec.g1_to_bytes(srs_mono[k])
        X = rng.integers(-128, 128, size=shape).astype(np.int8)
        coeffs = _fr_array(12)
        emu.interpolate(shape, X, T.TC_I8, coeffs)
        C = emu.commit(mono, coeffs, T.TC_FR)
        assert C == ec.g1_to_bytes(tc.commit_literal(pp, X)) == emu.commit(lag, X, T.TC_I8)
        kappa = (2, 1)
        yo, po = tc.open_literal(pp, X, kappa)
        rem = coeffs
        proof = []
        for axis in range(2):
            q, r = _fr_array(12), _fr_array(12)
            emu.divide_by_linear(shape, rem, axis, kappa[axis], q, r)
            proof.append(emu.commit(mono, q, T.TC_FR))
            rem = r
        assert proof == [ec.g1_to_bytes(p) for p in po]
        assert _fr_list(rem)[0] == yo and not any(_fr_list(rem)[1:])
        y, pi = emu.open(lag, X, T.TC_I8, kappa)        # the evaluation-form route gives the same proof
        assert pi == proof and y == ec.fr_to_bytes(yo)
        with pytest.raises(T.TcError) as err:
            emu.open(mono, X, T.TC_I8, kappa)
        assert err.value.code == T.binding.TC_ERR_STATE
        with pytest.raises(T.TcError):
            emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_MONOMIAL | T.TC_SRS_SUFFIX)
    finally:
        mono.close()
        lag.close()
    # argument errors
    with pytest.raises(T.TcError):
        emu.interpolate((2,) * 13, np.zeros(8192, dtype=np.int8), T.TC_I8, _fr_array(8192))
    with pytest.raises(T.TcError):
        emu.divide_by_linear((3, 4), coeffs, 2, 0, _fr_array(12), _fr_array(12))
    with pytest.raises(T.TcError):
        emu.divide_by_linear((3, 4), coeffs, 1, 4, _fr_array(12), _fr_array(12))
    with pytest.raises(T.TcError):
        emu.divide_by_linear((3, 4), coeffs, 1, 0, coeffs, _fr_array(12))


def test_emulated_incremental_update(emu, node_srs):
    """One entry changes: the library moves the commitments on its path only; the result must be the tree the
    oracle builds from scratch over the changed payload -- every node, and the openings after the update."""
    node, grid = (2, 2), (5, 7)
    X = tc_inputs.int16_uniform(grid, 9)
    tree = emu.terkle_build_entries(node_srs, X, T.TC_I16, grid, node)
    vk = emu.vk_from_trapdoor(TAU_BYTES)
    try:
        for leaf, new in (((3, 4), -32768), ((0, 0), 32767), ((4, 6), 0), ((3, 4), 5)):
            delta = int(new) - int(X[leaf])
            X[leaf] = new                                     # the caller's buffer
            tree.update(leaf, delta)
            ot = terkle.build(pps, tc.as_flat_ints(X), grid, node)
            for L in range(tree.levels):
                g, n = tree.level_info(L)
                for i in range(n):
                    assert tree.node(L, i) == ec.g1_to_bytes(ot.levels[L]["C"][tc.multi_index(i, g)]), (leaf, L, i)
            assert tree.root == ec.g1_to_bytes(ot.root)
            proof = tree.open(leaf)
            assert proof == serialize_steps(terkle.open_path(pps, ot, grid, node, leaf))
            assert emu.verify_path(vk, tree.path(leaf), tree.root, ec.fr_to_bytes(int(new) % R), proof)
        with pytest.raises(T.TcError):
            tree.update((5, 0), 1)
        with pytest.raises(T.TcError):
            tree.update((0, 0), 1 << 32)
    finally:
        tree.close()
    # a tensors tree: an entry inside a leaf tensor changes
    shapes = [(2, 3), (4,), (2, 2, 2), (3, 2)]
    rng = np.random.default_rng(17)
    leaves = [rng.integers(-50, 50, size=s).astype(np.int8) for s in shapes]
    srs = [emu.setup_from_trapdoor(TAU_BYTES, s, T.TC_SRS_SUFFIX) for s in shapes]
    tree = emu.terkle_build_tensors(node_srs, srs, leaves, [T.TC_I8] * 4, (2, 2), node)
    try:
        leaves[2][1, 0, 1] += 9
        tree.update((1, 0), 9, inner_index=(1, 0, 1))
        ot = terkle.build(pps, [tc.as_flat_ints(t) for t in leaves], (2, 2), node, kind="tensors", leaf_shapes=shapes)
        assert tree.root == ec.g1_to_bytes(ot.root)
        for i in range(4):
            assert tree.node(0, i) == ec.g1_to_bytes(ot.levels[0]["C"][tc.multi_index(i, (2, 2))])
        proof = tree.open((1, 0), (1, 0, 1))
        assert proof == serialize_steps(terkle.open_path(pps, ot, (2, 2), node, (1, 0), (1, 0, 1)))
        with pytest.raises(T.TcError):
            tree.update((1, 0), 1)                            # inner index missing
    finally:
        tree.close()
        for s in srs:
            s.close()


def test_emulated_tree_with_a_large_upper_level(emu, node_srs):
    """A level of more than 512 nodes above the bottom takes the four-wave node kernel with packed halving steps."""
    node, grid = (2, 2), (96, 100)
    X = tc_inputs.int8_uniform(grid, 5)
    tree = emu.terkle_build_entries(node_srs, X, T.TC_I8, grid, node)
    try:
        ot = terkle.build(pps, tc.as_flat_ints(X), grid, node)
        g1, n1 = tree.level_info(1)
        assert n1 > 512
        for L in (1, 2):
            g, n = tree.level_info(L)
            for i in list(range(0, n, 37)) + [n - 1]:
                assert tree.node(L, i) == ec.g1_to_bytes(ot.levels[L]["C"][tc.multi_index(i, g)]), (L, i)
        assert tree.root == ec.g1_to_bytes(ot.root)
    finally:
        tree.close()


def test_emulated_commit_static(emu):
    """The entry point that allocates nothing, on the host-emulation build: same bytes as tc_commit on a tensor of
    several tiles and then on a smaller one (the scratch keeps the first call's contents), a degenerate tensor whose
    single bucket needs every planned pass, no allocation by the library during the calls, the maximum size within
    the static scratch, and the limits refused with an error."""
    lib = emu.lib
    big, small = (96, 131), (7, 33)
    srs_big = emu.setup_from_trapdoor(TAU_BYTES, big, 0)
    srs_small = emu.setup_from_trapdoor(TAU_BYTES, small, 0)
    Xb = tc_inputs.int16_uniform(big, 21, -32768, 32767)
    Xs8 = tc_inputs.int8_uniform(small, 22)
    want_big, want_small = emu.commit(srs_big, Xb, T.TC_I16), emu.commit(srs_small, Xs8, T.TC_I8)
    same = np.full(big, 3, np.int16)                      # one bucket holds all 12576 terms
    want_same = emu.commit(srs_big, same, T.TC_I16)
    out = np.zeros(96, np.uint8)
    before = emu.alloc_calls()
    for srs, X, dt, want in ((srs_big, Xb, T.TC_I16, want_big), (srs_small, Xs8, T.TC_I8, want_small),
                             (srs_big, same, T.TC_I16, want_same), (srs_small, Xs8, T.TC_I8, want_small)):
        out[:] = 0xEE
        emu.commit_static(srs, X, dt, out)
        assert out.tobytes() == want
    assert emu.alloc_calls() == before, "tc_commit_static allocated or released memory"
    # errors: full-width scalars, a misaligned output, a tensor beyond the limit
    fr = fr_bytes_array([1] * (7 * 33))
    with pytest.raises(T.TcError) as e:
        emu.commit_static(srs_small, fr, T.TC_FR, out)
    assert e.value.code == T.binding.TC_ERR_ARG
    with pytest.raises(T.TcError) as e:
        emu.commit_static(srs_small, Xs8, T.TC_I8, out.ctypes.data + 1)
    assert e.value.code == T.binding.TC_ERR_ARG
    srs_big.close()
    srs_small.close()


@pytest.mark.slow
def test_emulated_commit_static_at_its_limit(emu):
    """TC_STATIC_MAX_TERMS int16 entries fit the static scratch (the call would fail with TC_ERR_NOMEM otherwise) and
    one entry more is refused.  The SRS of the emulation is slow to generate, so both tables are 1-D slices."""
    n = T.binding.TC_STATIC_MAX_TERMS
    srs = emu.setup_from_trapdoor(TAU_BYTES, (n,), 0)
    X = tc_inputs.int16_uniform((n,), 23, -32768, 32767)
    out = np.zeros(96, np.uint8)
    emu.commit_static(srs, X, T.TC_I16, out)
    assert out.tobytes() == emu.commit(srs, X, T.TC_I16)
    srs.close()
    srs = emu.setup_from_trapdoor(TAU_BYTES, (n + 1,), 0)
    with pytest.raises(T.TcError) as e:
        emu.commit_static(srs, np.zeros(n + 1, np.int16), T.TC_I16, out)
    assert e.value.code == T.binding.TC_ERR_SHAPE and "TC_STATIC_MAX_TERMS" in str(e.value)
    srs.close()


def test_emulated_srs_and_tree_files(emu, node_srs):
    """The public parameters and a built tree as flat files (Def. 4.1 Setup publishes pp; a tree is opened long
    after it was built): export -> import gives an SRS with the same points, commitments and openings, and a tree
    whose openings are the oracle's; damaged files are refused with an error code."""
    B = T.binding
    shape = (3, 4, 2)
    pp = pps(shape)
    srs = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    data = srs.export()
    n_pts = 24 + 8 + 2
    assert len(data) == 56 + 96 * n_pts and data[:5] == b"TCSRS"
    # the stored points are the oracle's Lagrange SRS and its suffix tables, canonical bytes
    S0 = pp.srs_lagrange(0)
    assert data[56 : 56 + 96 * 24] == b"".join(ec.g1_to_bytes(S0[i]) for i in range(24))
    assert data[56 + 96 * 32 :] == b"".join(ec.g1_to_bytes(p) for p in pp.srs_lagrange(2))
    back = emu.srs_import(data)
    assert back.shape == shape and back.size(0) == 24 and back.size(1) == 8 and back.size(2) == 2
    X = tc_inputs.int16_uniform(shape, 5, -32768, 32767)
    assert emu.commit(back, X, T.TC_I16) == ec.g1_to_bytes(tc.commit(pp, X))
    y, pi = emu.open(back, X, T.TC_I16, (2, 1, 1))          # needs the grid constants, which the import rebuilds
    yo, po = tc.open_(pp, X, (2, 1, 1))
    assert y == ec.fr_to_bytes(yo) and pi == [ec.g1_to_bytes(p) for p in po]
    assert all(back.point(i, a) == srs.point(i, a) for a, n in ((0, 24), (1, 8), (2, 2)) for i in range(n))
    back.close()
    # a monomial SRS and one without suffix tables keep their kind
    mono = emu.setup_from_trapdoor(TAU_BYTES, (3, 2), T.TC_SRS_MONOMIAL)
    mono2 = emu.srs_import(mono.export())
    assert mono2.flags == T.TC_SRS_MONOMIAL and [mono2.point(i) for i in range(6)] == [mono.point(i) for i in range(6)]
    with pytest.raises(T.TcError) as e:
        emu.open(mono2, np.zeros((3, 2), np.int8), T.TC_I8, (0, 0))
    assert e.value.code == B.TC_ERR_STATE
    mono.close()
    mono2.close()

    def refused(blob, code):
        with pytest.raises(T.TcError) as e:
            emu.srs_import(blob)
        assert e.value.code == code, (e.value.code, code)

    refused(data[:40], B.TC_ERR_ARG)                          # no complete header
    refused(data[:-1], B.TC_ERR_ARG)                          # truncated
    refused(data + b"\0", B.TC_ERR_ARG)                       # too long
    refused(b"XCSRS" + data[5:], B.TC_ERR_ARG)                # magic
    refused(data[:8] + (2).to_bytes(4, "little") + data[12:], B.TC_ERR_ARG)       # version
    refused(data[:12] + (7).to_bytes(4, "little") + data[16:], B.TC_ERR_ARG)      # curve
    refused(data[:48] + (n_pts - 1).to_bytes(8, "little") + data[56:], B.TC_ERR_ARG)      # count
    refused(data[:28] + (0).to_bytes(4, "little") + data[32:], B.TC_ERR_SHAPE)    # shape
    refused(data[:20] + (64).to_bytes(4, "little") + data[24:], B.TC_ERR_ARG)     # unknown flag
    off = 56 + 96 * 5
    refused(data[:off] + bytes([data[off] ^ 1]) + data[off + 1 :], B.TC_ERR_RANGE)         # a point off the curve
    refused(data[:off] + b"\xff" * 48 + data[off + 48 :], B.TC_ERR_RANGE)                   # x >= p
    srs.close()

    # a tree: built, saved, loaded, opened -- byte for byte the oracle's proofs
    node, grid = (2, 2), (5, 7)
    P = tc_inputs.int16_uniform(grid, 7)
    tree = emu.terkle_build_entries(node_srs, P, T.TC_I16, grid, node)
    blob = tree.export()
    ot = terkle.build(pps, tc.as_flat_ints(P), grid, node)
    n_nodes = sum(int(np.prod(lv["grid"])) for lv in ot.levels)
    assert len(blob) == 72 + 96 * n_nodes and blob[:6] == b"TCTREE"
    assert blob[-96:] == ec.g1_to_bytes(ot.root)
    root = tree.root
    tree.close()
    loaded = emu.terkle_build_entries(node_srs, P, T.TC_I16, grid, node, from_file=blob)
    assert loaded.root == root == ec.g1_to_bytes(ot.root) and loaded.levels == 3
    for leaf in [(0, 0), (4, 6), (2, 3)]:
        assert loaded.open(leaf) == serialize_steps(terkle.open_path(pps, ot, grid, node, leaf))
    loaded.update((1, 1), 3)                                # a loaded tree is a full tree: updates work on it
    P2 = P.copy()
    P2[1, 1] += 3
    assert loaded.root == ec.g1_to_bytes(terkle.build(pps, tc.as_flat_ints(P2), grid, node).root)
    loaded.close()
    for bad, code in ((blob[:-96], B.TC_ERR_ARG), (blob[:50], B.TC_ERR_ARG), (b"TCSRS\0\0\0" + blob[8:], B.TC_ERR_ARG),
                      (blob[:20] + (6).to_bytes(4, "little") + blob[24:], B.TC_ERR_SHAPE),
                      (blob[:72] + bytes([blob[72] ^ 1]) + blob[73:], B.TC_ERR_RANGE)):
        with pytest.raises(T.TcError) as e:
            emu.terkle_build_entries(node_srs, P, T.TC_I16, grid, node, from_file=bad)
        assert e.value.code == code, (e.value.code, code)
    # a tensors tree keeps its leaf commitments too
    shapes = [(2, 3), (4,), (2, 2, 2), (3, 3), (5,), (2, 2)]
    leaves = [tc_inputs.int16_uniform(s, 50 + i) for i, s in enumerate(shapes)]
    lsrs = [emu.setup_from_trapdoor(TAU_BYTES, s, T.TC_SRS_SUFFIX) for s in shapes]
    t2 = emu.terkle_build_tensors(node_srs, lsrs, leaves, [T.TC_I16] * 6, (3, 2), node)
    blob2 = t2.export()
    proof = t2.open((1, 0), (1, 0, 1))
    t2.close()
    l2 = emu.terkle_build_tensors(node_srs, lsrs, leaves, [T.TC_I16] * 6, (3, 2), node, from_file=blob2)
    assert l2.open((1, 0), (1, 0, 1)) == proof
    with pytest.raises(T.TcError) as e:                     # a file of an entries tree is not a tensors tree
        emu.terkle_build_tensors(node_srs, lsrs, leaves, [T.TC_I16] * 6, (3, 2), node, from_file=blob)
    assert e.value.code == B.TC_ERR_SHAPE
    l2.close()
    for s in lsrs:
        s.close()


def test_emulated_quant_scale(emu):
    """The per-tensor scale on the device side of the boundary: bit-equal to the oracle's float32(32767) / amax on
    tensors of several pieces and ragged ends, at any alignment, all zeros, a single outlier, subnormals,
    infinities and NaNs left out; and the quantisation that reads the scale from device memory."""
    from oracle import quantize

    rng = np.random.default_rng(3)
    cases = []
    for n in (1, 7, 8, 9, 1000, 8 * 256 * 3 + 5):
        cases.append(rng.standard_normal(n).astype(np.float16))
    cases.append(np.zeros(100, np.float16))
    outlier = (rng.standard_normal(5000) * 0.01).astype(np.float16)
    outlier[4321] = np.float16(-977.5)
    cases.append(outlier)
    cases.append(np.array([6e-8, -1.2e-7, 0.0], np.float16))                  # subnormals only
    mixed = rng.standard_normal(300).astype(np.float16)
    mixed[[3, 77]] = [np.inf, -np.inf]
    mixed[150] = np.nan
    cases.append(mixed)
    cases.append(np.array([np.inf, np.nan], np.float16))
    for x in cases:
        for offset in (0, 1, 3):                                             # elements past a 16-byte boundary
            store = np.zeros(x.size + 16, np.float16)
            view = store[offset : offset + x.size]
            view[:] = x
            out = np.full(1, -1.0, np.float32)
            emu.quant_scale(view, x.size, out)
            finite = x[np.isfinite(x)]
            want = quantize.inv_scale_for(finite) if finite.size else np.float32(0)
            assert out.view(np.uint32)[0] == np.float32(want).view(np.uint32), (x.size, offset, out[0], want)
            q = np.zeros(x.size, np.int16)
            emu.encode_tensor_scaled(view, T.TC_F16, x.size, out, q)
            ref = quantize.quantize_f16(np.where(np.isfinite(x), x, np.float16(0)), want)
            fin = np.isfinite(x)
            assert np.array_equal(q[fin], ref[fin])
    # the same tensors through the launches that all of them share, at mixed alignments, an empty one among them
    cases.append(np.zeros(0, np.float16))
    stores = [np.zeros(x.size + 16, np.float16) for x in cases]
    views = []
    for i, (x, st) in enumerate(zip(cases, stores)):
        v = st[i % 4 : i % 4 + x.size]
        v[:] = x
        views.append(v)
    outs = [np.full(x.size + 9, 77, np.int16) for x in cases]
    dsts = [o[(8 if i % 2 else 1) : (8 if i % 2 else 1) + x.size] for i, (x, o) in enumerate(zip(cases, outs))]
    scales = np.full(len(cases) + 2, -1.0, np.float32)
    emu.encode_batch_scaled(views, [x.size for x in cases], scales[1:], dsts)
    assert scales[0] == -1.0 and scales[-1] == -1.0
    for i, x in enumerate(cases):
        fin = np.isfinite(x)
        want = quantize.inv_scale_for(x[fin]) if fin.any() else np.float32(0)
        assert scales[1 + i : 2 + i].view(np.uint32)[0] == np.float32(want).view(np.uint32), i
        ref = quantize.quantize_f16(np.where(fin, x, np.float16(0)), want)
        assert np.array_equal(dsts[i][fin], ref[fin]), i
        lo = 8 if i % 2 else 1
        assert (outs[i][:lo] == 77).all() and (outs[i][lo + x.size :] == 77).all()
    with pytest.raises(T.TcError):
        emu.encode_batch_scaled([views[0]], [1 << 33], scales[1:], [dsts[0]])


def test_emulated_field_ops(emu):
    """The field-operation hook on the host build (the portable forms of the same routines) against Python
    integers: the check that the GPU test applies to the device forms, validated here without a GPU."""

    def run(op, a, b, words):
        out = np.zeros(a.size, np.uint32)
        emu.field_op(op, a, b, a.size // words, out)
        return out

    check_field_arithmetic(run, 200, 100)


def test_emulated_options(emu, monkeypatch):
    """Tuning options: refused outside their ranges, taken from the environment at context creation, and without
    effect on results -- the same int16 and full-width commitments under several plans of the accumulation."""
    B = T.binding
    for opt, bad in ((B.TC_OPT_ACC_SUBRUN, 65), (B.TC_OPT_ACC_SUBRUN, -1), (B.TC_OPT_ACC_FANIN, 1), (B.TC_OPT_FR_WINDOW, 12),
                     (B.TC_OPT_CHECK_LEVEL, 2), (17, 1)):
        with pytest.raises(T.TcError) as e:
            emu.set_option(opt, bad)
        assert e.value.code == B.TC_ERR_ARG
    assert [emu.get_option(o) for o in range(4)] == [0, 0, 0, 0]
    monkeypatch.setenv("TC_ACC_SUBRUN", "7")
    monkeypatch.setenv("TC_ACC_FANIN", "banana")
    monkeypatch.setenv("TC_FR_WINDOW", "9")
    other = T.Context(0, lib=emu.lib)
    assert [other.get_option(o) for o in range(4)] == [7, 0, 0, 0]
    other.close()
    shape = (16, 256)
    pp = pps(shape)
    srs = emu.setup_from_trapdoor(TAU_BYTES, shape, 0)
    X = tc_inputs.int16_uniform(shape, 21, -32768, 32767)
    X.reshape(-1)[:700] = 5                                    # one full bucket: several passes over its partial sums
    F = fr_bytes_array([(v * 0x1F3D5B79A2C4E6F1) % R for v in range(1, 16 * 256 + 1)])
    want16, wantfr = ec.g1_to_bytes(tc.commit(pp, X)), None
    try:
        for sub, fan, win in ((0, 0, 0), (1, 2, 8), (3, 5, 16), (64, 64, 0)):
            emu.set_option(B.TC_OPT_ACC_SUBRUN, sub)
            emu.set_option(B.TC_OPT_ACC_FANIN, fan)
            emu.set_option(B.TC_OPT_FR_WINDOW, win)
            emu.set_option(B.TC_OPT_CHECK_LEVEL, 1)
            assert emu.commit(srs, X, T.TC_I16) == want16, (sub, fan, win)
            got = emu.commit(srs, F, T.TC_FR)
            wantfr = wantfr or got
            assert got == wantfr, (sub, fan, win)
    finally:
        for o in range(4):
            emu.set_option(o, 0)
    srs.close()


def test_emulated_commit_over_repeated_points(emu):
    """Equal and opposite points inside the bucket sums (see check_repeated_points), on the host build."""
    check_repeated_points(emu, lambda a: a, many=8)
    check_one_point_throughout(emu, lambda a: a, (16, 128))


def test_emulated_open_with_the_opening_table(emu, node_srs):
    """TC_SRS_OPEN_TABLE: the table's points are U[kappa, t] = sum_(k != kappa) S[k, t] / (zeta_k - zeta_kappa) (checked
    against the oracle's group arithmetic on the Lagrange SRS), openings through it equal the oracle's byte for byte
    (int16 and int8, corner and interior positions, equal rows), the table survives export / import, and a tensors
    tree keeps the row commitments of a leaf between opening calls and drops them when the leaf is updated."""
    B = T.binding
    shape = (8, 2048)
    pp = pps(shape)
    srs = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX | T.TC_SRS_OPEN_TABLE)
    data = srs.export()
    assert len(data) == 56 + 96 * (2 * 8 * 2048 + 2048)
    # three entries of U from the definition, with the oracle's scalars: U[kappa, t] = [l_t(tau_2) sum_k l_k(tau_1) / (k - kappa)] G
    for kappa, t in ((0, 0), (5, 1000), (7, 2047)):
        g = sum(pp.ell[0][k] * ec.fr_inv(k - kappa) for k in range(8) if k != kappa) % R
        want = ec.mul(g * pp.ell[1][t] % R, ec.G1)
        off = 56 + 96 * (8 * 2048 + 2048 + kappa * 2048 + t)
        assert data[off : off + 96] == ec.g1_to_bytes(want)
    back = emu.srs_import(data)
    X16 = tc_inputs.int16_uniform(shape, 3, -32768, 32767)
    X16[0, 0], X16[7, 2047], X16[3, 77] = -32768, 32767, -32768
    X16[4, :] = X16[3, :]
    X8 = tc_inputs.int8_uniform(shape, 4)
    for s in (srs, back):
        for X, dt in ((X16, T.TC_I16), (X8, T.TC_I8)):
            for kappa in [(3, 77), (0, 0), (7, 2047)]:
                y, pi = emu.open(s, X, dt, kappa)
                yo, po = tc.open_(pp, X, kappa)
                assert y == ec.fr_to_bytes(yo) and pi == [ec.g1_to_bytes(p) for p in po]
    back.close()
    with pytest.raises(T.TcError) as e:
        emu.setup_from_trapdoor(TAU_BYTES, (64,), T.TC_SRS_OPEN_TABLE)
    assert e.value.code == B.TC_ERR_SHAPE
    # a tensors tree: two leaves share the shape; several openings per call and over several calls; then an update
    plain = emu.setup_from_trapdoor(TAU_BYTES, shape, T.TC_SRS_SUFFIX)
    leaves = [X16.copy(), tc_inputs.int16_uniform(shape, 8), tc_inputs.int16_uniform(shape, 9)]
    for lsrs in ([srs, srs, plain], [srs, srs, srs]):
        tree = emu.terkle_build_tensors(node_srs, lsrs, leaves, [T.TC_I16] * 3, (3, 1), (2, 2))
        ot_leaf = [tc.commit(pp, l) for l in leaves]
        otree = terkle.build(pps, [terkle.phi(c) for c in ot_leaf], (3, 1), (2, 2))

        def oracle_proof(leaf, inner, tensor):
            steps = terkle.open_path(pps, otree, (3, 1), (2, 2), leaf)
            k, y, pi, _ = steps[-1]
            steps[-1] = (k, y, pi, tc.commit(pp, tensor))
            yo, po = tc.open_(pp, tensor, inner)
            steps.append((inner, yo, po, None))
            return serialize_steps(steps)

        assert tree.root == ec.g1_to_bytes(otree.root)
        calls = [[((0, 0), (3, 77)), ((1, 0), (0, 5)), ((0, 0), (6, 2000)), ((2, 0), (2, 2))],     # leaf 0 twice in one call
                 [((0, 0), (1, 1)), ((1, 0), (7, 2047))]]                                          # later call: kept rows
        for batch in calls:
            got = tree.open_batch([b[0] for b in batch], [b[1] for b in batch])
            for (leaf, inner), proof in zip(batch, got):
                assert proof == oracle_proof(leaf, inner, leaves[leaf[0]]), (leaf, inner)
        # leaf 0 changes: its kept row commitments must not be used again
        leaves[0][6, 2000] += 5
        tree.update((0, 0), 5, (6, 2000))
        ot_leaf[0] = tc.commit(pp, leaves[0])
        otree = terkle.build(pps, [terkle.phi(c) for c in ot_leaf], (3, 1), (2, 2))
        assert tree.root == ec.g1_to_bytes(otree.root)
        assert tree.open((0, 0), (6, 1999)) == oracle_proof((0, 0), (6, 1999), leaves[0])
        leaves[0][6, 2000] -= 5
        tree.close()
    plain.close()
    srs.close()
