"""Writes tests/golden/c1_oracle.json from the CPU oracle alone (never from the HIP path).

Run:  python tests/golden/make_golden.py
The file stores, for the tiny configuration (one int8 tensor of shape (4,16,16), seed 0,
trapdoors from SHA-256 labels), the oracle's commitment and eight openings as canonical
bytes in hex.  The paper prints no worked numeric example, so these are regression
values of the oracle, not values taken from the paper."""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import tc_inputs  # noqa: E402
from oracle import bls12_381 as ec  # noqa: E402
from oracle import tc  # noqa: E402


def main():
    tau = tc_inputs.trapdoors()
    pp = tc.setup(tc_inputs.C1_SHAPE, tau)
    T = tc_inputs.c1_tensor()
    out = {
        "source": "oracle/tc.py closed-form routes; see make_golden.py",
        "shape": list(tc_inputs.C1_SHAPE),
        "commitment": ec.g1_to_bytes(tc.commit(pp, T)).hex(),
        "openings": [],
    }
    for kappa in tc_inputs.opening_positions(tc_inputs.C1_SHAPE, 8, tc_inputs.tensor_seed(0)):
        y, proof = tc.open_(pp, T, kappa)
        out["openings"].append(
            {"kappa": list(kappa), "y": ec.fr_to_bytes(y).hex(), "pi": [ec.g1_to_bytes(p).hex() for p in proof]}
        )
    with open(os.path.join(HERE, "c1_oracle.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
