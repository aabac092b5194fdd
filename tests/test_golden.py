import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_and_generator_reproduce_the_frozen_tiny_case():
    spec = importlib.util.spec_from_file_location("make_expected", os.path.join(HERE, "golden", "make_expected.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.compute()
    with open(os.path.join(HERE, "golden", "tiny_f32_expected.json")) as fh:
        want = json.load(fh)
    assert got["n_valid"] == want["n_valid"] and got["targets_first8"] == want["targets_first8"]
    for k in ("loss", "H_sum", "W_abs_sum", "dH_abs_max", "dW_abs_max", "dH_dot_H"):
        assert abs(got[k] - want[k]) <= 1e-10 * max(1.0, abs(want[k])), k
    np.testing.assert_allclose(got["lse_first4"], want["lse_first4"], rtol=1e-12)
