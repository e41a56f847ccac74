import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")
    config.addinivalue_line("markers", "slow: CPU test that takes more than a few seconds")
    # long tests report their progress past pytest's output capture (a run that prints nothing for minutes looks hung)
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import gpu_util

    gpu_util.CAPTURE_MANAGER = config.pluginmanager.getplugin("capturemanager")
