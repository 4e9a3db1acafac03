import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

_config = None


def pytest_configure(config):
    global _config
    _config = config
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_runtest_logreport(report):
    """Progress reaches the log as each test ends, also when stdout is a pipe or a file (a long GPU run that stays
    silent for minutes looks hung to whoever watches it)."""
    if report.when != "teardown" or _config is None:
        return
    tr = _config.pluginmanager.get_plugin("terminalreporter")
    tw = getattr(tr, "_tw", None)
    if tw is not None:
        try:
            tw.flush()
        except Exception:
            pass
