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


class Stopwatch:
    """Prints what a long test is doing and how long each part took (the GPU machine takes silence for a hang)."""

    def __init__(self, name):
        self.name, self.t0, self.last = name, time.time(), time.time()

    def lap(self, what):
        now = time.time()
        print("%s: %s (%.1f s, %.1f s since start)" % (self.name, what, now - self.last, now - self.t0), flush=True)
        self.last = now
