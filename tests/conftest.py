import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def alpha_table():
    """alpha*(b) as the oracle derives it (numeric minimisation), computed once per session."""
    from oracle import alpha_star
    return {b: alpha_star.alpha_star(b) for b in (1, 2, 3, 4, 8)}
