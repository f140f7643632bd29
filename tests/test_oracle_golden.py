"""The oracle still reproduces the stage digests stored for the Tiny
configuration (written by tests/golden/make_golden.py from the oracle alone)."""
import importlib.util
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_tiny_digests_unchanged():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = open(os.path.join(HERE, "golden", "tiny_oracle.txt")).read().splitlines()
    assert list(mod.lines()) == stored
