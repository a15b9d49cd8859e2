import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


from progress import set_capture_manager  # noqa: E402  (tests/ is on the path: pytest's rootdir insertion)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    set_capture_manager(config.pluginmanager.getplugin("capturemanager"))
