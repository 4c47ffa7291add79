"""The oracle still produces the frozen OPT-125m-linear fixture (written by
tests/golden/make_golden.py from the oracle alone; not a value from the paper)."""
import importlib.util
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_golden_fixture():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(HERE, "golden", "opt125m_linear_oracle.txt")) as f:
        assert mod.compute() == f.read()
