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
    import oracle as orc
    orc.lib()
    return orc


def pytest_terminal_summary(terminalreporter):
    """Lists the heads whose retained set differed from the oracle's at a near-tie and was
    accepted (layer, head, the cut that differed first, the oracle's gap there)."""
    try:
        from tests import util
    except Exception:
        return
    if util.EXCUSED:
        terminalreporter.write_line(f"index mismatches accepted at near-ties: {len(util.EXCUSED)}")
        for case in util.EXCUSED:
            terminalreporter.write_line(f"  {case}")
