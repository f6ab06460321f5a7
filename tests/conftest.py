import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_built():
    from oracle import build_oracle
    return build_oracle()


@pytest.fixture
def set_hook(monkeypatch):
    """Sets one of the library's environment hooks for the rest of the test: the library keeps
    what it read at its first call, so it is told to read the environment again, and once more
    when the variable has been restored."""
    import paper_2511_11939_amd as P

    def _set(name, value):
        monkeypatch.setenv(name, value)
        P.prism_reread_environment()

    yield _set
    monkeypatch.undo()
    P.prism_reread_environment()
