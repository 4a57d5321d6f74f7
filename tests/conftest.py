import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (runs the HIP library)")


_CONFIG = None


@pytest.hookimpl(trylast=True)
def pytest_sessionstart(session):
    global _CONFIG
    _CONFIG = session.config


def say(msg):
    """One line that names the GPU case about to run (test, shape, entry point) or reports what it measured,
    written past pytest's output capture and flushed, so that it is on the terminal before the GPU step starts."""
    line = f"[gpu-case] {msg}"
    pm = _CONFIG.pluginmanager if _CONFIG is not None else None
    tr = pm.get_plugin("terminalreporter") if pm is not None else None
    capman = pm.get_plugin("capturemanager") if pm is not None else None
    if tr is not None and capman is not None:
        with capman.global_and_fixture_disabled():
            tr.ensure_newline()
            tr.write_line(line)
            tr._tw.flush()
    else:
        print(line, file=sys.stderr, flush=True)
