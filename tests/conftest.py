import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # tests/test_oracle_mutations.py re-runs the pin files in a child process with one planted mistake
    # switched on; nothing is patched unless that variable is set
    mutant = os.environ.get("VTC_ORACLE_MUTANT")
    if mutant:
        from tests import mutants

        mutants.apply(mutant)


@pytest.fixture(scope="session")
def repo_root():
    return ROOT
