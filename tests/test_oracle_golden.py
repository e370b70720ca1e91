"""The oracle still reproduces its stored outputs on the tiny fixture case (regression guard; see tests/golden/README.md)."""
import importlib.util
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_fixture():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    ref = json.load(open(os.path.join(HERE, "golden", "oracle_tiny.json")))
    assert now["budgets"] == ref["budgets"] and now["indices_head0"] == ref["indices_head0"]
    for key in ("score_head0_first8", "smoothed_head0_first8", "score_sums"):
        np.testing.assert_allclose(now[key], ref[key], rtol=1e-12, atol=1e-15)
