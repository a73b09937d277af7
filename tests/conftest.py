import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


CAPTURE_MANAGER = None      # pytest's capture plugin: parity_util.announce() writes past it


def pytest_configure(config):
    global CAPTURE_MANAGER
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    CAPTURE_MANAGER = config.pluginmanager.getplugin("capturemanager")


@pytest.fixture(scope="session", autouse=True)
def _oracle_built():
    """The CPU checker is compiled once per session if its library is absent or stale."""
    from oracle import build_oracle
    build_oracle.build(force=False)
