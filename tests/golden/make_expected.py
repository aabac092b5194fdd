"""Writes tests/golden/tiny_f32_expected.json.

The paper prints no worked numeric example (its evaluation is a latency and
memory sweep), so there is no paper value to store.  This file instead freezes
what the CPU oracle returns on the seeded "tiny_f32" workload, so that an
accidental change to the input generator or to the oracle shows up as a diff.
It calls only oracle/ and the input generator; nothing here comes from the GPU.

    python tests/golden/make_expected.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import flce_oracle as O                      # noqa: E402
from paper_2511_17599_amd import inputs as I             # noqa: E402


def compute():
    wl = I.WORKLOADS["tiny_f32"]
    x = I.make_inputs(wl)
    H, W = I.to_f64(x["H"]), I.to_f64(x["W"])
    f = O.forward(H, W, x["y"], wl.ignore_index, wl.reduction)
    b = O.backward(H, W, x["y"], wl.ignore_index, wl.reduction)
    return {
        "workload": wl.name, "seed": wl.seed,
        "n_valid": f["n_valid"],
        "loss": f["loss"],
        "lse_first4": [float(v) for v in f["lse"][:4]],
        "targets_first8": [int(v) for v in x["y"][:8]],
        "H_sum": float(H.sum()), "W_abs_sum": float(np.abs(W).sum()),
        "dH_abs_max": float(np.abs(b["dH"]).max()), "dW_abs_max": float(np.abs(b["dW"]).max()),
        "dH_dot_H": float((b["dH"] * H).sum()),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_f32_expected.json")
    with open(out, "w") as fh:
        json.dump(compute(), fh, indent=1)
        fh.write("\n")
    print("wrote", out)
