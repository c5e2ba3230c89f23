import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import kvev_oracle
    kvev_oracle.build()
    return kvev_oracle


def pytest_terminal_summary(terminalreporter):
    """Parity figures the tests measured (kept-index comparison, worst errors): printed at any verbosity."""
    from tests import helpers
    if helpers.REPORTS:
        terminalreporter.section("parity report")
        for line in helpers.REPORTS:
            terminalreporter.write_line(line)
