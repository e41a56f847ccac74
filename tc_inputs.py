"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds NO arithmetic of the method (no field, curve, commitment or
tree code): only random tensors of the workloads' shapes and value
distributions, the trapdoor seeds and the opening positions.  Both the CPU
oracle's tests and the GPU tests draw their inputs from here so that the two
sides see the same data.

Workloads (stand-ins for the paper's LLaMA-2 activations and weights, which
are not available): C1 tiny int8 tensor (4,16,16); C2 one 512 x 4096 fp16
N(0,1) activation; C3 a LLaMA2-7B-shaped forward (32 layers x {512x4096,
512x4096, 512x11008}); C4 LLaMA2-7B-shaped int8 weights; C5 LLaMA2-13B-shaped
batched activations.
"""
import hashlib

import numpy as np

# BLS12-381 group order, needed only to reduce the hashed trapdoor seeds.
_R = 0x73EDA753299D7D483339D80809A1D80553BDA402FFFE5BFEFFFFFFFF00000001

MAX_ORDER = 4


def trapdoors(m=MAX_ORDER, label="tc/trapdoor/v1/"):
    """tau_j = SHA-256(label || str(j)) mod r, j = 0..m-1 (test-only trusted setup)."""
    return [int.from_bytes(hashlib.sha256((label + str(j)).encode()).digest(), "big") % _R for j in range(m)]


def trapdoor_bytes(m=MAX_ORDER, label="tc/trapdoor/v1/"):
    return b"".join(int(t).to_bytes(32, "little") for t in trapdoors(m, label))


def tensor_seed(cfg, req=0, layer=0, kind=0):
    return cfg * 10**6 + req * 10**4 + layer * 10 + kind


def int8_uniform(shape, seed, lo=-128, hi=127):
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int8)


def int16_uniform(shape, seed, lo=-32767, hi=32767):
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int16)


def f16_normal(shape, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(size=shape, dtype=np.float32).astype(np.float16)


def opening_positions(shape, count, seed):
    rng = np.random.default_rng(seed + 999)
    return [tuple(int(rng.integers(0, d)) for d in shape) for _ in range(count)]


# --- the five configurations --------------------------------------------------
C1_SHAPE = (4, 16, 16)
C2_SHAPE = (512, 4096)
NODE_SHAPE = (4, 4)                      # "arity 16"
LLAMA7B = dict(layers=32, tokens=512, hidden=4096, mlp=11008)
LLAMA13B = dict(layers=40, tokens=2048, hidden=5120, mlp=13824, batch=8)


def c1_tensor():
    return int8_uniform(C1_SHAPE, tensor_seed(0))


def c2_activation(shape=C2_SHAPE):
    return f16_normal(shape, tensor_seed(1))


def c3_shapes(cfg=LLAMA7B):
    """Per layer: residual output, attention output, MLP intermediate."""
    t, h, f = cfg["tokens"], cfg["hidden"], cfg["mlp"]
    return [(t, h), (t, h), (t, f)]


def c4_shapes(cfg=LLAMA7B):
    """Per layer: Wq, Wk, Wv, Wo, W_gate, W_up, W_down."""
    h, f = cfg["hidden"], cfg["mlp"]
    return [(h, h)] * 4 + [(h, f)] * 2 + [(f, h)]
