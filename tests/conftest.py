import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    try:                                     # progress lines of the long GPU tests bypass the capture (tests/gpu_util.say)
        from tests import gpu_util
        gpu_util._capture_manager = config.pluginmanager.getplugin("capturemanager")
    except Exception:                        # no torch / no library on this machine: the GPU tests are not run anyway
        pass


@pytest.fixture(scope="session", autouse=True)
def _oracle_built():
    from oracle.build_oracle import build
    build(force=False)
