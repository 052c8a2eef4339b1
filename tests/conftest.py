import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden(name):
    """Parse a tests/golden/*.txt fixture: '#' lines are comments (they carry the citation),
    every other non-empty line is 'key value [value ...]'."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, *vals = line.split()
            out[key] = vals
    return out


_CONFIG = None


def pytest_sessionstart(session):
    global _CONFIG
    _CONFIG = session.config


def progress(msg: str) -> None:
    """One line to the real stdout, past pytest's capture: long GPU tests report each stage, so that a run that
    is merely busy can be told from one that hangs."""
    line = "[gpu-test] " + msg
    capman = _CONFIG.pluginmanager.getplugin("capturemanager") if _CONFIG is not None else None
    if capman is None:
        print(line, flush=True)
        return
    with capman.global_and_fixture_disabled():
        print(line, flush=True)
