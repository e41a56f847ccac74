"""CPU oracle for the TensorCommitments prover path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct
implementation of what the path computes, written from the paper's
definitions (Def. 2.2, Def. 4.1, the Terkle Tree definitions, Algorithm 1,
App. C).  It shares no code with the HIP library and never imports it.  Only
`tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py`
may use it; the product path must never route through it.

Modules
  bls12_381  the field/curve layer (Python ints; App. E: curve, group law)
  tc         Setup / Com / Open / Ver of Def. 4.1 (three commit routes, three
             opening routes, trapdoor-form verification)
  terkle     Terkle Tree build, membership proof, path verification
  quantize   float -> integer -> field embedding used by the synthetic workloads
  cbind      ctypes binding of the plain-C oracle (`c/tc_oracle.c`): naive
             double-and-add MSM and closed-form field sums at sizes Python
             cannot reach in seconds

Parity unpinned by the paper (the paper is silent; fixed by this build's own
readings): the integer grid nodes, the map G1 -> Fr for internal tree nodes,
the quantisation rule, the tree shapes, zero padding, byte encodings.
"""
