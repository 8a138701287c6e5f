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
    from oracle import ws_oracle
    ws_oracle.build()
    return ws_oracle


@pytest.fixture
def say(capsys):
    """Print past pytest's capture.  The full-size GPU tests run for minutes and report each head as it is checked;
    their lines go straight to the terminal, so a watcher of the run sees progress while a test is under way."""
    def line(text):
        with capsys.disabled():
            print(text, flush=True)
    return line
