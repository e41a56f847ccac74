"""Quantisation and field embedding used by the synthetic workloads -- oracle.

TEST INFRASTRUCTURE ONLY.  The paper treats tensors as already lying in F^{d_1 x..x d_m}
(Sec. 3) and never says how floating-point activations get there; this rule is
this build's reading (parity unpinned by the paper):

    q = clamp(rint(float32(x) * inv_scale), -32767, 32767)     (round half to even)
    e(q) = q if q >= 0 else r - |q|

with inv_scale = float32(32767) / float32(max|x|) computed once per tensor in
float32 by the caller (0 if the tensor is all zeros) and passed to both sides.
The product is a single float32 multiply (no fused multiply-add is involved).
"""
import numpy as np

from .bls12_381 import R

QMAX = 32767


def inv_scale_for(x):
    """float32(32767) / float32(amax); 0.0 for an all-zero tensor."""
    amax = np.float32(np.max(np.abs(np.asarray(x, dtype=np.float32)))) if np.asarray(x).size else np.float32(0)
    if amax == 0:
        return np.float32(0.0)
    return np.float32(np.float32(QMAX) / amax)


def quantize_f16(x, inv_scale):
    """fp16 array -> int16 array, elementwise, by the rule above."""
    x32 = np.asarray(x, dtype=np.float16).astype(np.float32)
    prod = (x32 * np.float32(inv_scale)).astype(np.float32)
    q = np.rint(prod)                               # numpy rint rounds half to even
    q = np.clip(q, -QMAX, QMAX)
    return q.astype(np.int16)


def embed(q):
    return int(q) % R
