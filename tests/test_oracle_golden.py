"""The oracle still reproduces the digests stored by tests/golden/make_golden.py
(a regression guard written by the oracle alone; the paper prints no values)."""
import importlib.util
import json
import os

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
mg = importlib.util.module_from_spec(spec)
spec.loader.exec_module(mg)

with open(os.path.join(HERE, "golden", "oracle_digests.json")) as f:
    STORED = json.load(f)


@pytest.mark.parametrize("case", mg.CASES, ids=[c[0] for c in mg.CASES])
def test_oracle_reproduces_stored_digests(oracle, case):
    assert mg.run_case(case) == STORED[case[0]]
