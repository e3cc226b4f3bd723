import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
if os.path.dirname(os.path.abspath(__file__)) not in sys.path:
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    import gpu_util
    gpu_util.PYTEST_CONFIG = config


@pytest.fixture(scope="session")
def oracle_nn():
    """The oracle's C layers, built on demand (gcc, a second or two)."""
    from oracle import build, nn
    so = os.path.join(ROOT, "oracle", "liboracle_nn.so")
    src = os.path.join(ROOT, "oracle", "nn_layers.c")
    if not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
        build.build()
    return nn
