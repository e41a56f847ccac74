"""Pins for the oracle's Terkle Tree and quantisation (CPU only)."""
import numpy as np
import pytest

import tc_inputs
from oracle import bls12_381 as ec
from oracle import quantize, tc, terkle
from oracle.bls12_381 import P, R

TAU = tc_inputs.trapdoors()
_cache = {}


def pps(shape):
    shape = tuple(shape)
    if shape not in _cache:
        _cache[shape] = tc.setup(shape, TAU)
    return _cache[shape]


def test_phi_map():
    assert terkle.phi(ec.INF) == 0
    a = ec.mul(999, ec.G1)
    assert terkle.phi(a) != terkle.phi(ec.neg(a))                   # separates C from -C
    x, y = a
    big = y > (P - 1) // 2
    assert terkle.phi(a) == (2 * x + (1 if big else 0)) % R
    assert (terkle.phi(a) - terkle.phi(ec.neg(a))) % R in (1, R - 1)


def test_entries_tree_shape_root_and_paths():
    grid, node = (6, 10), (4, 4)
    X = tc_inputs.int16_uniform(grid, 7)
    tree = terkle.build(pps, tc.as_flat_ints(X), grid, node)
    # level grids: ceil(6/4, 10/4) = (2,3) -> (1,1); every in-range node is built
    assert [lv["grid"] for lv in tree.levels] == [(2, 3), (1, 1)]
    assert [len(lv["C"]) for lv in tree.levels] == [6, 1]
    # a bottom node commits its zero-padded block
    Z, shape = tree.levels[0]["Z"][(1, 2)]
    block = np.zeros((4, 4), np.int64)
    block[:2, :2] = X[4:6, 8:10]
    assert Z == [int(v) for v in block.reshape(-1)] and shape == node
    assert tree.levels[0]["C"][(1, 2)] == tc.commit(pps(node), block)
    # the root commits phi of the six children and zeros elsewhere
    Zr, _ = tree.levels[1]["Z"][(0, 0)]
    for k1 in range(4):
        for k2 in range(4):
            want = terkle.phi(tree.levels[0]["C"][(k1, k2)]) if (k1 < 2 and k2 < 3) else 0
            assert Zr[k1 * 4 + k2] == want
    assert tree.root == tc.commit(pps(node), Zr)
    for leaf in [(0, 0), (5, 9), (3, 4)]:
        steps = terkle.open_path(pps, tree, grid, node, leaf)
        assert len(steps) == 2                                      # one opening per level
        shapes = [node] * 2
        assert terkle.verify_path(pps, tree.root, shapes, int(X[leaf]), steps)
        assert not terkle.verify_path(pps, tree.root, shapes, int(X[leaf]) + 1, steps)
        assert not terkle.verify_path(pps, ec.add(tree.root, ec.G1), shapes, int(X[leaf]), steps)
        # wrong child commitment
        k, y, pi, child = steps[0]
        bad = [(k, y, pi, ec.add(child, ec.G1))] + steps[1:]
        assert not terkle.verify_path(pps, tree.root, shapes, int(X[leaf]), bad)
        # wrong proof element at the bottom
        k, y, pi, child = steps[1]
        bad = [steps[0], (k, y, [pi[0], ec.add(pi[1], ec.G1)], child)]
        assert not terkle.verify_path(pps, tree.root, shapes, int(X[leaf]), bad)


def test_flipped_entry_changes_every_ancestor():
    grid, node = (8, 8), (2, 2)
    X = tc_inputs.int16_uniform(grid, 3)
    t1 = terkle.build(pps, tc.as_flat_ints(X), grid, node)
    assert [lv["grid"] for lv in t1.levels] == [(4, 4), (2, 2), (1, 1)]
    assert [len(lv["C"]) for lv in t1.levels] == [16, 4, 1]
    X2 = X.copy()
    X2[5, 2] ^= 1
    t2 = terkle.build(pps, tc.as_flat_ints(X2), grid, node)
    chain = terkle.path_indices(t1, grid, node, (5, 2))
    on_path = {(lvl, a) for lvl, a, _ in chain}
    for lvl, lv in enumerate(t1.levels):
        for a, C in lv["C"].items():
            assert (t2.levels[lvl]["C"][a] != C) == ((lvl, a) in on_path)
    steps = terkle.open_path(pps, t1, grid, node, (5, 2))
    assert not terkle.verify_path(pps, t2.root, [node] * 3, int(X[5, 2]), steps)


def test_tensors_tree():
    grid, node = (3, 2), (2, 2)
    shapes = [(2, 3), (4,), (2, 2, 2), (3, 3), (5,), (2, 2)]
    leaves = [tc_inputs.int16_uniform(s, 50 + i) for i, s in enumerate(shapes)]
    tree = terkle.build(pps, [tc.as_flat_ints(t) for t in leaves], grid, node, kind="tensors", leaf_shapes=shapes)
    assert [lv["grid"] for lv in tree.levels] == [(3, 2), (2, 1), (1, 1)]
    for i, t in enumerate(leaves):
        assert tree.levels[0]["C"][tc.multi_index(i, grid)] == tc.commit(pps(shapes[i]), t)
    inner = (1, 0, 1)
    steps = terkle.open_path(pps, tree, grid, node, (1, 0), inner)       # tensor (1,0) is leaves[2]
    assert len(steps) == 3
    sh = [node, node, shapes[2]]
    assert terkle.verify_path(pps, tree.root, sh, int(leaves[2][inner]), steps)
    assert not terkle.verify_path(pps, tree.root, sh, int(leaves[2][inner]) + 1, steps)
    # roots of different payloads differ
    leaves2 = [t.copy() for t in leaves]
    leaves2[4][0] += 1
    tree2 = terkle.build(pps, [tc.as_flat_ints(t) for t in leaves2], grid, node, kind="tensors", leaf_shapes=shapes)
    assert tree2.root != tree.root


def test_single_node_tree_is_one_tc():
    X = tc_inputs.c1_tensor()
    tree = terkle.build(pps, tc.as_flat_ints(X), (4, 16, 16), (4, 16, 16))
    assert len(tree.levels) == 1 and tree.root == tc.commit(pps((4, 16, 16)), X)
    for leaf in tc_inputs.opening_positions((4, 16, 16), 2, 0):
        steps = terkle.open_path(pps, tree, (4, 16, 16), (4, 16, 16), leaf)
        assert len(steps) == 1 and len(steps[0][2]) == 3
        assert terkle.verify_path(pps, tree.root, [(4, 16, 16)], int(X[leaf]), steps)


def test_c2b_level_counts():
    """Uniform (4,4) tree over a 512 x 4096 grid: 6 levels, 139 813 nodes (counts only)."""
    g = (512, 4096)
    counts = []
    g = terkle.ceil_div_shape(g, (4, 4))
    counts.append(g[0] * g[1])
    while any(x > 1 for x in g):
        g = terkle.ceil_div_shape(g, (4, 4))
        counts.append(g[0] * g[1])
    assert counts == [131072, 8192, 512, 32, 4, 1] and sum(counts) == 139813


def test_quantize_rule():
    inv = np.float32(2.0)
    x = np.array([0.25, 0.75, 1.25, -0.25, -0.75, 1.0, -1.0, 0.0, 60000.0, -60000.0], np.float16)
    q = quantize.quantize_f16(x, inv)
    # products 0.5, 1.5, 2.5, -0.5, -1.5 round half to even; large values clamp
    assert q.tolist() == [0, 2, 2, 0, -2, 2, -2, 0, 32767, -32767]
    assert q.dtype == np.int16
    a = tc_inputs.f16_normal((64, 64), 3)
    s = quantize.inv_scale_for(a)
    qa = quantize.quantize_f16(a, s)
    assert int(np.max(np.abs(qa))) == 32767
    assert s == np.float32(32767.0) / np.float32(np.max(np.abs(a.astype(np.float32))))
    assert quantize.inv_scale_for(np.zeros(4, np.float16)) == 0
    assert quantize.quantize_f16(np.zeros(4, np.float16), 0.0).tolist() == [0, 0, 0, 0]
    assert quantize.embed(-5) == R - 5 and quantize.embed(7) == 7 and tc.embed(-128) == R - 128


def test_golden_c1_matches_oracle():
    import json
    import os

    with open(os.path.join(os.path.dirname(__file__), "golden", "c1_oracle.json")) as f:
        gold = json.load(f)
    pp = pps(tuple(gold["shape"]))
    T = tc_inputs.c1_tensor()
    assert ec.g1_to_bytes(tc.commit(pp, T)).hex() == gold["commitment"]
    C = ec.g1_from_bytes(bytes.fromhex(gold["commitment"]))
    for o in gold["openings"]:
        y = ec.fr_from_bytes(bytes.fromhex(o["y"]))
        pi = [ec.g1_from_bytes(bytes.fromhex(h)) for h in o["pi"]]
        assert tc.verify(pp, C, tuple(o["kappa"]), y, pi)
        assert y == int(T[tuple(o["kappa"])]) % R


def test_node_over_zeros_has_the_identity_as_commitment_and_still_verifies():
    """A node whose tensor is all zero commits to the identity; it enters its parent as phi(O) = 0, and a path
    through it must still verify (the child carried by the proof is the identity, not a missing child)."""
    grid, node = (4, 4), (2, 2)
    X = np.arange(16).reshape(grid) + 1
    X[2:4, 2:4] = 0
    tree = terkle.build(pps, tc.as_flat_ints(X), grid, node)
    assert tree.levels[0]["C"][(1, 1)] is ec.INF
    leaf = (3, 2)
    steps = terkle.open_path(pps, tree, grid, node, leaf)
    assert steps[0][3] is ec.INF and steps[0][1] == 0            # the top step opens phi(O) = 0 and carries O
    assert terkle.verify_path(pps, tree.root, [node] * 2, 0, steps)
    assert not terkle.verify_path(pps, tree.root, [node] * 2, 1, steps)
    moved = [(steps[0][0], steps[0][1], steps[0][2], ec.G1)] + steps[1:]
    assert not terkle.verify_path(pps, tree.root, [node] * 2, 0, moved)
