import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    if not config.pluginmanager.hasplugin("timeout"):
        # the per-test limit is pytest-timeout's; without the plugin the mark is only a label
        config.addinivalue_line("markers", "timeout(seconds): per-test time limit")
