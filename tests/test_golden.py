"""The stored Tiny fixture (written by tests/golden/make_tiny_golden.py from the oracle alone)
still matches what the oracle computes, and has the properties the definitions fix."""
import importlib.util
import json
import os

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


def _load_variants():
    spec = importlib.util.spec_from_file_location("make_variants_golden", os.path.join(HERE, "golden", "make_variants_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracle_reproduces_the_stored_tiny_lamb_step():
    mod = _load_variants()
    want = json.load(open(os.path.join(HERE, "golden", "tiny_lamb_step.json")))
    got = mod.compute_lamb()
    assert got["status"] == want["status"] == 0 and got["coefs"] == want["coefs"]
    assert got["norms"] == pytest.approx(want["norms"], rel=1e-14)
    assert got["trust"] == pytest.approx(want["trust"], rel=1e-13)
    for a, b in zip(got["tensors"], want["tensors"]):
        for k in ("p", "m", "v"):
            assert a[k] == pytest.approx(b[k], rel=1e-13, abs=0)
        assert a["p_sum"] == pytest.approx(b["p_sum"], rel=1e-11)
    assert want["coefs"][0] < 1 and all(t > 0 and t != 1.0 for t in want["trust"])


def test_load_balancing_oracle_reproduces_the_stored_small_table():
    mod = _load_variants()
    want = json.load(open(os.path.join(HERE, "golden", "small_lbs_table.json")))
    assert mod.compute_lbs() == want                  # integers: exact
    m = want["methods"]
    rng = {k: m[k]["sum_max"] - m[k]["sum_min"] for k in m}
    assert rng["none"] > rng["stratified"] > rng["local_raster"] > rng["local_snake"]
    assert all(6 * 1 + 3 * 129 + 2 * 257 + 5 * 385 <= x for x in m["stratified"]["trial_min"])   # the quota's lower bound
    d = want["first_draws_gpu0_trial0"]
    assert [(x - 1) // 128 for x in d] == [0] * 6 + [1] * 3 + [2] * 2 + [3] * 5
