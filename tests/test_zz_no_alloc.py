"""GPU test of tc_commit_static, the entry point that allocates nothing (for callers that cannot call hipMalloc:
code under graph capture, tight serving loops).  Through the C ABI: its output must equal tc_commit's byte for byte
(integer work: no tolerance) and the oracle's closed form, on calls in a row that share the device's static
scratch array -- the largest tensor it takes, then smaller ones -- and the library must not have allocated or
released anything meanwhile."""
import numpy as np
import pytest

import tc_inputs
from oracle import bls12_381 as ec
from oracle import cbind

from gpu_util import TAU_BYTES, pps, to_device

pytestmark = pytest.mark.gpu


def test_commit_static_matches_commit_on_calls_in_a_row():
    import torch

    import paper_2602_12630_amd as T

    assert torch.cuda.is_available(), "the GPU tests need a GPU"
    B = T.binding
    ctx = T.Context(0)
    big = (64, 4096)                                     # TC_STATIC_MAX_TERMS entries: a 64-token slab of a 4096-wide activation
    small = (37, 501)                                    # ragged tiles, int8
    assert big[0] * big[1] == B.TC_STATIC_MAX_TERMS
    srs_big = ctx.setup_from_trapdoor(TAU_BYTES, big, 0)
    srs_small = ctx.setup_from_trapdoor(TAU_BYTES, small, 0)
    rng = np.random.default_rng(tc_inputs.tensor_seed(1, 0, 0, 7))
    Xb = np.clip(np.rint(rng.standard_normal(big) * 6000.0), -32767, 32767).astype(np.int16)     # quantised N(0,1): bell-shaped bucket loads
    Xs = tc_inputs.int8_uniform(small, 31)
    Xc = np.full(big, -5, np.int16)                      # one bucket holds every term: all planned passes do real work
    cases = [(srs_big, Xb, T.TC_I16), (srs_small, Xs, T.TC_I8), (srs_big, Xc, T.TC_I16), (srs_small, Xs, T.TC_I8)]
    dev = [to_device(X) for _, X, _ in cases]
    want = [ctx.commit(srs, d, dt) for (srs, _, dt), d in zip(cases, dev)]
    outs = [torch.full((96,), 0xEE, dtype=torch.uint8, device="cuda") for _ in cases]
    torch.cuda.synchronize()
    before = ctx.alloc_calls()
    for (srs, _, dt), d, out in zip(cases, dev, outs):   # back to back on one stream, nothing waited for in between
        ctx.commit_static(srs, d, dt, out)
    after = ctx.alloc_calls()
    ctx.sync()
    got = [bytes(out.cpu().numpy().tobytes()) for out in outs]
    assert after == before, "tc_commit_static allocated or released device / pinned memory"
    for i, (g, w) in enumerate(zip(got, want)):
        assert g == w, "call %d differs from tc_commit" % i
    # and against the oracle's closed form (the small tensor in full, the constant one as [c] G)
    assert got[1] == ec.g1_to_bytes(cbind.commit(pps(small), Xs))
    assert got[2] == ec.g1_to_bytes(cbind.g1_mul(-5 % ec.R, ec.G1))
    # limits are refused with a clear error, not run
    srs_over = ctx.setup_from_trapdoor(TAU_BYTES, (big[0] * big[1] + 1,), 0)
    over = torch.zeros(big[0] * big[1] + 1, dtype=torch.int16, device="cuda")
    with pytest.raises(T.TcError) as e:
        ctx.commit_static(srs_over, over, T.TC_I16, outs[0])
    assert e.value.code == B.TC_ERR_SHAPE and "TC_STATIC_MAX_TERMS" in str(e.value)
    with pytest.raises(T.TcError) as e:
        ctx.commit_static(srs_small, dev[1], T.TC_FR, outs[0])
    assert e.value.code == B.TC_ERR_ARG
    for s in (srs_big, srs_small, srs_over):
        s.close()
    ctx.close()
