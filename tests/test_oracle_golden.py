"""The CPU checker still reproduces the values frozen under tests/golden/ (written by
tests/golden/make_golden.py from oracle/ alone; the paper prints no worked example)."""
import importlib.util
import json
import os

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_config1_values_are_reproduced():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = json.load(open(os.path.join(HERE, "golden", "config1_chain.json")))
    now = mod.compute()
    assert sorted(now) == sorted(stored)
    for k, v in stored.items():
        assert now[k] == pytest.approx(v, rel=1e-12), k
