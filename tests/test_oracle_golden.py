"""The frozen small case under tests/golden/ (written by make_golden.py from the oracle alone)."""
import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_frozen_small_case(oracle):
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    k, cu, hq, hkv, d, Q, K, V, dO = mg.make_case()
    with open(os.path.join(HERE, "golden", "ttt_small_case.json")) as f:
        g = json.load(f)
    assert (g["k"], g["cu_seqlens"], g["hq"], g["hkv"], g["d"]) == (k, cu, hq, hkv, d)
    got = oracle.oracle_full(Q, K, V, cu, g["scale"], dO)
    for name, x in zip(("O", "LSE", "dQ", "dK", "dV"), got):
        np.testing.assert_allclose(x, np.array(g[name]), rtol=0, atol=1e-13, err_msg=name)
