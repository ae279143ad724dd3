import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")
    config.addinivalue_line("markers", "slow: takes more than a few seconds of CPU time")
    # harness.progress() suspends the capture for its one line (looked up there through this attribute)
    pytest.bagel_capture_manager = config.pluginmanager.getplugin("capturemanager")


def pytest_runtest_logstart(nodeid, location):
    # one flushed line per test on the real stderr: with the output piped (block-buffered dots) a run of
    # several long tests would otherwise print nothing for minutes
    sys.__stderr__.write(f"[test] {nodeid}\n")
    sys.__stderr__.flush()
