import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # test_oracle_mutants.py re-runs the oracle's pins in a child process with one planted
    # mistake switched on through this variable; it is never set otherwise
    mutant = os.environ.get("CURDKV_ORACLE_MUTANT")
    if mutant:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from oracle_mutants import MUTANTS
        MUTANTS[mutant]()


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
