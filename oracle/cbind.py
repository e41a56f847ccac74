"""ctypes binding of the plain-C oracle (`oracle/c/tc_oracle.c`).  TEST INFRASTRUCTURE ONLY."""
import ctypes
import os
import subprocess

import numpy as np

from . import bls12_381 as ec

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "c", "tc_oracle.c")
LIB = os.path.join(_HERE, "c", "libtc_oracle.so")

I8, I16, FR = 1, 2, 3
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (building the checker is not using it)."""
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread", "-o", LIB, SRC])
    return LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(LIB)
        L.tco_init.restype = ctypes.c_int
        L.tco_msm_naive.restype = ctypes.c_int
        L.tco_msm_naive.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                    ctypes.c_void_p]
        L.tco_f_at_tau.restype = ctypes.c_int
        L.tco_f_at_tau.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.c_int, ctypes.c_void_p]
        L.tco_init()
        _lib = L
    return _lib


def _kind_of(arr):
    if arr.dtype == np.int8:
        return I8
    if arr.dtype == np.int16:
        return I16
    raise TypeError("scalars must be int8 / int16 arrays or Fr byte strings")


def _buf(b):
    return (ctypes.c_uint8 * len(b)).from_buffer_copy(b)


def fr_mul(a, b):
    out = (ctypes.c_uint8 * 32)()
    lib().tco_fr_mul(_buf(ec.fr_to_bytes(a)), _buf(ec.fr_to_bytes(b)), out)
    return int.from_bytes(bytes(out), "little")


def fp_mul(a, b):
    out = (ctypes.c_uint8 * 48)()
    lib().tco_fp_mul(_buf(int(a).to_bytes(48, "little")), _buf(int(b).to_bytes(48, "little")), out)
    return int.from_bytes(bytes(out), "little")


def fp_inv(a):
    out = (ctypes.c_uint8 * 48)()
    lib().tco_fp_inv(_buf(int(a).to_bytes(48, "little")), out)
    return int.from_bytes(bytes(out), "little")


def g1_add(a, b):
    out = (ctypes.c_uint8 * 96)()
    lib().tco_g1_add(_buf(ec.g1_to_bytes(a)), _buf(ec.g1_to_bytes(b)), out)
    return ec.g1_from_bytes(bytes(out))


def g1_mul(k, pt):
    out = (ctypes.c_uint8 * 96)()
    lib().tco_g1_mul(_buf(ec.fr_to_bytes(k % ec.R)), _buf(ec.g1_to_bytes(pt)), out)
    return ec.g1_from_bytes(bytes(out))


def g1_generator():
    out = (ctypes.c_uint8 * 96)()
    lib().tco_g1_generator(out)
    return ec.g1_from_bytes(bytes(out))


def msm_naive(scalars, points_bytes, nthreads=1):
    """scalars: int8/int16 numpy array, or bytes of 32-byte Fr values; points_bytes: n x 96 bytes.
    Returns (point, threads_used)."""
    if isinstance(scalars, (bytes, bytearray)):
        n = len(scalars) // 32
        kind = FR
        sbuf = _buf(bytes(scalars))
        sptr = ctypes.addressof(sbuf)
    else:
        arr = np.ascontiguousarray(scalars).reshape(-1)
        n = arr.size
        kind = _kind_of(arr)
        sptr = arr.ctypes.data
    assert len(points_bytes) == 96 * n
    pbuf = _buf(bytes(points_bytes))
    out = (ctypes.c_uint8 * 96)()
    used = lib().tco_msm_naive(sptr, kind, ctypes.addressof(pbuf), n, int(nthreads), out)
    return ec.g1_from_bytes(bytes(out)), used


def f_at_tau(T, shape, ell, nthreads=1):
    """sum_i e(T[i]) prod_j ell[j][i_j] mod r for an int8/int16 numpy tensor."""
    arr = np.ascontiguousarray(T).reshape(-1)
    shape = [int(d) for d in shape]
    assert arr.size == int(np.prod(shape, dtype=np.int64))
    ell_bytes = b"".join(ec.fr_to_bytes(v) for axis in ell for v in axis)
    ebuf = _buf(ell_bytes)
    sh = (ctypes.c_uint32 * len(shape))(*shape)
    out = (ctypes.c_uint8 * 32)()
    rc = lib().tco_f_at_tau(arr.ctypes.data, _kind_of(arr), len(shape), sh, ctypes.addressof(ebuf), int(nthreads), out)
    if rc != 0:
        raise ValueError("bad shape")
    return int.from_bytes(bytes(out), "little")


def commit(pp, T, nthreads=1):
    """C_T = [f_T(tau)] G with the field sum and the scalar multiplication both in C."""
    return g1_mul(f_at_tau(T, pp.shape, pp.ell, nthreads), ec.G1)


def open_(pp, T, kappa, nthreads=1):
    """Open (Def. 4.1) under a known trapdoor, the same closed form as tc.open_: R_i = r_i(tau) is the slice of T
    with its first i indices fixed to kappa, contracted with the Lagrange values of the remaining axes;
    q_i(tau) = (R_{i-1} - R_i) / (tau_i - omega_i); pi_i = [q_i(tau)] G.  The field sums and the scalar
    multiplications run in C (large int8 / int16 tensors); returns (y, [pi_1 .. pi_m])."""
    kappa = tuple(int(k) for k in kappa)
    if len(kappa) != pp.m or any(not (0 <= k < d) for k, d in zip(kappa, pp.shape)):
        raise ValueError("opening index outside the grid")
    sub = np.ascontiguousarray(T).reshape(pp.shape)
    Rs = []
    for i in range(pp.m):
        Rs.append(f_at_tau(sub, pp.shape[i:], pp.ell[i:], nthreads))
        sub = sub[kappa[i]]
    Rs.append(int(sub) % ec.R)
    proof = []
    for i in range(pp.m):
        omega_i = kappa[i] + 1                       # the grid node of position kappa_i
        q = (Rs[i] - Rs[i + 1]) * ec.fr_inv(pp.tau[i] - omega_i) % ec.R
        proof.append(g1_mul(q, ec.G1))
    return Rs[pp.m], proof
