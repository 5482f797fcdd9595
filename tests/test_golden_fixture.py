"""The CPU oracle still produces the digests frozen in tests/golden/ (the fixture is written
by tests/golden/make_golden.py from the oracle alone; the paper prints no worked example).
A failure here means the oracle's arithmetic or conventions moved: justify it with the
paper, then regenerate the fixture."""
import importlib.util
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_the_frozen_digests():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = [l.rstrip("\n") for l in open(os.path.join(HERE, "golden", "oracle_config1_batch.txt")) if not l.startswith("#")]
    assert mod.compute() == stored
