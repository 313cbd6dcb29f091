"""Regression guard: the oracle still produces the digests recorded for workload 1
(tests/golden/config1_oracle_digest.json, written by tests/golden/make_golden.py from
oracle/ alone).  A change to the oracle's arithmetic shows up here and must be justified."""
import importlib.util
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_config1_digests_unchanged():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(HERE, "golden", "config1_oracle_digest.json")) as f:
        want = json.load(f)
    assert mod.digests() == want
