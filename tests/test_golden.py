"""The stored Tiny fixture (written by tests/golden/make_tiny_golden.py from the oracle alone)
still matches what the oracle computes, and has the properties the definitions fix."""
import importlib.util
import json
import math
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _load():
    spec = importlib.util.spec_from_file_location("make_tiny_golden", os.path.join(HERE, "golden", "make_tiny_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod, json.load(open(os.path.join(HERE, "golden", "tiny_fused_step.json")))


def test_oracle_reproduces_the_stored_tiny_step():
    mod, want = _load()
    got = mod.compute()
    assert got["status"] == want["status"] == 0
    assert got["norms"] == pytest.approx(want["norms"], rel=1e-14)
    assert got["coefs"] == want["coefs"]
    for a, b in zip(got["tensors"], want["tensors"]):
        for k in ("g", "p", "m", "v"):
            assert a[k] == pytest.approx(b[k], rel=1e-13, abs=0)
        for k in ("p_sum", "m_sum", "v_sum"):
            assert a[k] == pytest.approx(b[k], rel=1e-11)


def test_stored_values_obey_the_step_one_closed_form():
    # from m = v = 0 at t = 1:  m' = (1-b1) ghat, v' = (1-b2) ghat^2 with ghat = coef * g
    _, want = _load()
    assert want["coefs"][0] < 1 and want["coefs"][1] == 1.0 and want["coefs"][2] == 1.0
    assert want["coefs"][0] == pytest.approx(0.1 / want["norms"][0], rel=1e-7)
    for coef, t in zip(want["coefs"], want["tensors"]):
        for g, m, v in zip(t["g"], t["m"], t["v"]):
            assert m == pytest.approx(0.1 * coef * g, rel=1e-12)
            assert v == pytest.approx(0.001 * (coef * g) ** 2, rel=1e-12)
