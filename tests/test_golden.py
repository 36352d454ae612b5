"""Regression guard of the oracles: tests/golden/oracle_regression.json (written by
tests/golden/make_golden.py from oracle/ only) must still be what the oracles produce."""
import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def _close(a, b):
    if isinstance(a, list):
        assert len(a) == len(b)
        for x, y in zip(a, b):
            _close(x, y)
    elif isinstance(a, int):
        assert a == b
    else:
        assert abs(a - b) <= 1e-9 * max(1.0, abs(b)), (a, b)


def test_oracle_outputs_match_the_stored_fixture():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.compute()
    want = json.load(open(os.path.join(HERE, "golden", "oracle_regression.json")))
    assert sorted(got) == sorted(want)
    for case in want:
        assert sorted(got[case]) == sorted(want[case])
        for key in want[case]:
            _close(got[case][key], want[case][key])
    # sanity of the fixture itself: softmax gradients sum to zero over the vocabulary; masks keep something
    assert want["lmhead_config0"]["dW_colsum_max"] < 1e-12
    assert min(want["dynakv_tiny"]["k"]) >= 1 and np.isfinite(want["dynakv_tiny"]["xbar_fro"])
