"""Drift guard: the oracle and the input generator still reproduce the stored tiny case."""
import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_tiny_case_matches_stored_oracle_output(oracle):
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    with open(os.path.join(HERE, "golden", "tiny_oracle.json")) as fh:
        stored = json.load(fh)
    for key, val in stored.items():
        if isinstance(val, str):
            continue
        np.testing.assert_allclose(np.asarray(now[key]), np.asarray(val), rtol=1e-9, atol=1e-15, err_msg=key)
