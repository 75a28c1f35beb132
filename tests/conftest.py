import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


_CFG_CACHE = {}


@pytest.fixture(scope="session")
def cfg():
    """cfg(i, num_layers=None) -> cached synthetic configuration i."""
    import ffsynth

    def get(i, num_layers=None):
        key = (i, num_layers)
        if key not in _CFG_CACHE:
            _CFG_CACHE[key] = ffsynth.make_config(i, num_layers=num_layers)
        return _CFG_CACHE[key]
    return get
