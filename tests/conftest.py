import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


_CONFIG = None


def pytest_configure(config):
    global _CONFIG
    _CONFIG = config
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def progress(msg: str):
    """Print a progress line past pytest's output capture (a long oracle run must not look hung to
    whoever watches the run's output), and into the captured output as well."""
    print(msg, flush=True)
    capman = _CONFIG.pluginmanager.getplugin("capturemanager") if _CONFIG is not None else None
    if capman is not None and capman.is_globally_capturing():
        with capman.global_and_fixture_disabled():
            print(msg, flush=True)


def load_golden(name):
    """Parse a `key: v v v` text fixture under tests/golden/ into {key: [int, ...]}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":", 1)
            out[key.strip()] = [int(x) for x in vals.split()]
    return out


@pytest.fixture(scope="session")
def worked_example():
    return load_golden("worked_example.txt")
