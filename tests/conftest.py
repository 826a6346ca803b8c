import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def lgo():
    from oracle import lgo as _lgo
    alt = os.environ.get("LGO_ORACLE_LIB")      # a mutant build, see test_oracle_mutants.py
    if alt:
        return _lgo.Oracle(alt)
    _lgo.lib()
    return _lgo
