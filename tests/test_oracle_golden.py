"""The oracle still reproduces the frozen small-case fixture."""
import importlib.util
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_matches_frozen_fixture():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(HERE, "golden", "oracle_small.txt")) as f:
        lines = [ln.split() for ln in f if not ln.startswith("#")]
    assert len(lines) == len(mod.CASES)
    for tok in lines:
        cid = int(tok[0])
        _, O = mod.compute(cid)
        np.testing.assert_allclose(O[0, 0, -1], np.array([float(x) for x in tok[1:]]), rtol=1e-13, atol=1e-15)
