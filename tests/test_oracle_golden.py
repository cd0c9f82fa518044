"""The oracle's whole run on the tiny workload against the stored digest (tests/golden/tiny_run.json,
written by tests/golden/make_golden.py from the oracle alone): guards the oracle against unintended
change.  Its formulas are pinned elsewhere (closed forms, invariants, brute force)."""
import importlib.util
import json
import os

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _load_maker():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.mark.parametrize("idx,threshold", [(0, 0.8), (1, -2.0)])
def test_tiny_run_matches_stored_digest(idx, threshold):
    with open(os.path.join(HERE, "golden", "tiny_run.json")) as f:
        want = json.load(f)["runs"][idx]
    got = _load_maker().run(threshold)
    assert got["events"] == want["events"]
    assert got["final_log_S_sum"] == pytest.approx(want["final_log_S_sum"], abs=1e-5)
    for g, w in zip(got["outputs_sum_abs_first_last"], want["outputs_sum_abs_first_last"]):
        assert g == pytest.approx(w, rel=1e-7, abs=1e-8)
