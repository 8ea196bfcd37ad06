"""The oracle against its own recorded results (tests/golden/oracle_regression.json, written by
tests/golden/make_oracle_fixtures.py from the oracle alone).  Not a pin - the pins are in
test_oracle_*_pins.py - but a guard: the oracle's arithmetic does not change unnoticed."""
import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def _load_maker():
    spec = importlib.util.spec_from_file_location("make_oracle_fixtures", os.path.join(HERE, "golden", "make_oracle_fixtures.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracle_reproduces_its_recorded_results():
    with open(os.path.join(HERE, "golden", "oracle_regression.json")) as f:
        want = json.load(f)
    got = _load_maker().cases()
    # integers, tokens, decisions: exact
    assert got["forward"]["prompt"] == want["forward"]["prompt"]
    for r, w in want["forward"]["rows"].items():
        g = got["forward"]["rows"][r]
        assert g["argmax"] == w["argmax"]
        np.testing.assert_allclose(g["first8"], w["first8"], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(g["sum"], w["sum"], rtol=1e-9, atol=1e-9)
    for key in ("draft", "n_accepted", "next"):
        assert got["accept"][key] == want["accept"][key]
    np.testing.assert_allclose(got["accept"]["p_row0_first4"], want["accept"]["p_row0_first4"], rtol=1e-9)
    assert got["loop"] == want["loop"]
    # the recorded run exercises both outcomes of the rejection step
    assert 0 < sum(want["loop"]["accepted"]) < 3 * len(want["loop"]["accepted"])
    assert any(a < 4 for a in want["accept"]["n_accepted"])
