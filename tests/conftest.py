import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    # tests/test_oracle_mutations.py re-runs the pin files against oracle builds with a planted
    # mistake: it points this variable at the mutant's shared library (CPU only)
    mutant = os.environ.get("ORACLE_MUTANT_LIB")
    if mutant:
        oracle._LIB = mutant
    oracle.build()
    return oracle
