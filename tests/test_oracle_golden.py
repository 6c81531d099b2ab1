"""The oracle reproduces its stored results on tiny seeded inputs (a guard against silent changes of its
arithmetic; the values come from tests/golden/make_golden.py, which calls only the oracle)."""
import importlib.util
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_matches_its_stored_results():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = json.loads(json.dumps(mod.build()))
    stored = json.load(open(os.path.join(HERE, "golden", "oracle_regression.json")))
    assert sorted(now) == sorted(stored)
    for key in stored:
        a, b = now[key], stored[key]
        assert len(a) == len(b), key
        for x, y in zip(a, b):
            if isinstance(y, float):
                assert abs(x - y) <= 1e-9 * max(1.0, abs(y)), key
            else:
                assert x == y, key
