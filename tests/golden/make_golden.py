"""Writes tests/golden/c1_oracle_digest.json: digests of what the CPU oracle computes for the tiny
configuration (128 x 512 -> 512).  Calls only the oracle and the seeded input generator; nothing
here comes from the HIP library.  The paper prints no numeric worked example of the quantized
linear layer, so this fixture pins the oracle against drift, not against the paper.

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import linear as oracle            # noqa: E402
import fptq_workloads as synth         # noqa: E402


def digests():
    out = {}
    for case in synth.config_cases("c1"):
        inp = synth.draw(case)
        ref = oracle.w4a4_linear(inp.x_bits, inp.w_int, inp.s_a, inp.s_w, case.mode, case.eps)
        out[case.name] = {k: hashlib.sha256(np.ascontiguousarray(ref[k]).tobytes()).hexdigest() for k in ("r", "q", "acc", "y")}
        out[case.name]["s_a_bits"] = int(np.float32(inp.s_a).view(np.uint32))
        out[case.name]["acc_abs_max"] = int(np.abs(ref["acc"]).max())
        out[case.name]["q_histogram"] = np.bincount(ref["q"].ravel().astype(np.int64) + 8, minlength=16).tolist()
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle_digest.json")
    with open(path, "w") as f:
        json.dump(digests(), f, indent=1)
    print("wrote", path)
