import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    mutant = os.environ.get("PG_ORACLE_MUTANT")
    if mutant:        # set only by test_oracle_pins_catch_mistakes.py for its child sessions
        from oracle import pg_oracle
        from tests._oracle_mutants import plant
        plant(pg_oracle, mutant)


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
