"""Terkle Tree: build, membership proof, path verification -- oracle.

TEST INFRASTRUCTURE ONLY.  Follows the Terkle Tree definitions of Sec. 4: every
node u gathers its children in a tensor Z_u (payload entries at the bottom,
child commitments above), stores C_u = Com_TC(Z_u); the root commitment is C_r;
a membership proof is one TC opening per level; the verifier walks the path,
checks every opening, that each opened value matches the next commitment on the
path, and that the top commitment is the root.

Readings where the paper is silent (parity unpinned by the paper):
  * a child commitment enters Z_u through phi: G1 -> Fr,
        phi(O) = 0,  phi(C) = (2 x_C + s(y_C)) mod r,  s(y) = 1 iff y > (p-1)/2,
    on canonical affine coordinates;
  * a tree is a payload grid plus one node shape per level; the grid of level
    l+1 is ceil(grid_l / node_shape_l) per axis (spatial blocking); children
    outside the grid are the field element 0;
  * the bottom level is either blocks of payload entries ("entries" tree) or
    whole tensors, one TC each with its own shape ("tensors" tree);
  * the proof carries, besides the openings, the commitments of the nodes on
    the path below the root (the verifier needs them to check the match).
"""
from . import bls12_381 as ec
from . import tc
from .bls12_381 import P, R


def phi(C):
    if C is ec.INF:
        return 0
    x, y = C
    return (2 * x + (1 if y > (P - 1) // 2 else 0)) % R


def ceil_div_shape(grid, node_shape):
    return tuple(-(-g // d) for g, d in zip(grid, node_shape))


class Tree:
    """levels[l] = dict(grid, node_shape (None for whole-tensor leaves), Z: {a: flat values},
    C: {a: commitment}); level 0 is the bottom, the last level holds the root."""

    def __init__(self):
        self.levels = []
        self.kind = None

    @property
    def root(self):
        top = self.levels[-1]
        (c,) = top["C"].values()
        return c


def _block(values, grid, node_shape, a):
    """Z for node `a`: the node_shape block of `values` (flat, shape `grid`) at block index a,
    zero outside the grid."""
    out = []
    for f in range(tc.prod(node_shape)):
        k = tc.multi_index(f, node_shape)
        g = tuple(ai * d + ki for ai, d, ki in zip(a, node_shape, k))
        if all(gi < n for gi, n in zip(g, grid)):
            out.append(values[tc.flat_index(g, grid)])
        else:
            out.append(0)
    return out


def build(pps, payload, grid, node_shape, kind="entries", leaf_shapes=None):
    """Recursive build.

    pps: function shape -> PublicParams (one trapdoor vector for the whole context).
    kind == "entries": `payload` is the flat integer tensor of shape `grid`.
    kind == "tensors": `payload` is a list (row-major over `grid`) of flat integer
        tensors, leaf_shapes[i] the shape of tensor i; the bottom level is one TC
        per tensor.
    node_shape: the node shape used at every blocked level (same order m as grid).
    """
    grid = tuple(int(g) for g in grid)
    node_shape = tuple(int(d) for d in node_shape)
    tree = Tree()
    tree.kind = kind

    # the level grids, bottom-up
    if kind == "entries":
        level_grids = [ceil_div_shape(grid, node_shape)]
    else:
        level_grids = [grid]
    while any(g > 1 for g in level_grids[-1]):
        level_grids.append(ceil_div_shape(level_grids[-1], node_shape))
    if kind == "tensors" and len(level_grids) == 1 and tc.prod(grid) == 1:
        pass                                         # a single tensor: the leaf TC is the root
    for lg in level_grids:
        tree.levels.append({"grid": lg, "node_shape": node_shape, "Z": {}, "C": {}})
    if kind == "tensors":
        tree.levels[0]["node_shape"] = None

    def node(level, a):
        lv = tree.levels[level]
        if a in lv["C"]:
            return lv["C"][a]
        if level == 0 and kind == "tensors":
            i = tc.flat_index(a, grid)
            Z = [int(v) for v in payload[i]]
            shape = tuple(leaf_shapes[i])
        elif level == 0:
            Z = _block(payload, grid, node_shape, a)
            shape = node_shape
        else:
            below = tree.levels[level - 1]["grid"]
            Z = []
            for f in range(tc.prod(node_shape)):
                k = tc.multi_index(f, node_shape)
                g = tuple(ai * d + ki for ai, d, ki in zip(a, node_shape, k))
                if all(gi < n for gi, n in zip(g, below)):
                    Z.append(phi(node(level - 1, g)))
                else:
                    Z.append(0)
            shape = node_shape
        C = tc.commit(pps(shape), Z)
        lv["Z"][a] = (Z, shape)
        lv["C"][a] = C
        return C

    top = len(tree.levels) - 1
    node(top, tuple(0 for _ in grid))
    # a recursive build from the root reaches every in-range node
    return tree


def path_indices(tree, grid, node_shape, leaf):
    """For a payload position, the node index and child multi-index at every blocked level,
    bottom-up.  `leaf` is the payload grid multi-index (entries tree) or the tensor's
    grid multi-index (tensors tree)."""
    out = []
    pos = tuple(int(x) for x in leaf)
    first = 0 if tree.kind == "entries" else 1
    for level in range(first, len(tree.levels)):
        a = tuple(p // d for p, d in zip(pos, node_shape))
        k = tuple(p % d for p, d in zip(pos, node_shape))
        out.append((level, a, k))
        pos = a
    return out


def open_path(pps, tree, grid, node_shape, leaf, inner=None):
    """Membership proof, top level first.  Each step: (kappa, y, [pi_1..pi_m], C_child)
    where C_child is the commitment of the next node down the path (None at the bottom).
    For a tensors tree `inner` is the multi-index of the entry inside the leaf tensor."""
    steps = []
    chain = path_indices(tree, grid, node_shape, leaf)
    for level, a, k in reversed(chain):
        Z, shape = tree.levels[level]["Z"][a]
        y, pi = tc.open_(pps(shape), Z, k)
        if level > 0:
            child_idx = tuple(ai * d + ki for ai, d, ki in zip(a, node_shape, k))
            child = tree.levels[level - 1]["C"][child_idx]
        else:
            child = None
        steps.append((k, y, pi, child))
    if tree.kind == "tensors":
        a = tuple(int(x) for x in leaf)
        Z, shape = tree.levels[0]["Z"][a]
        y, pi = tc.open_(pps(shape), Z, inner)
        steps.append((tuple(inner), y, pi, None))
    return steps


def verify_path(pps, root, shapes, leaf_value, steps):
    """shapes[d] = node shape at step d (top first).  Accept iff every opening verifies
    against the commitment carried down the path, every opened value at an internal
    step equals phi(child commitment), the bottom value is the claimed leaf value and
    the chain starts at the root."""
    if len(shapes) != len(steps):
        return False
    C = root
    for d, (kappa, y, pi, child) in enumerate(steps):
        if not tc.verify(pps(shapes[d]), C, kappa, y, pi):
            return False
        last = d == len(steps) - 1
        if last:
            if y != leaf_value % R:
                return False
        else:
            # the child may be the identity (a node over zeros only): phi(O) = 0, and INF is None here
            if y != phi(child):
                return False
            C = child
    return True
