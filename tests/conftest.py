import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


_CAPTURE = None


def pytest_configure(config):
    global _CAPTURE
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    _CAPTURE = config.pluginmanager.getplugin("capturemanager")


def progress(msg: str) -> None:
    """One line about a finished step of a long test (an oracle pass over 2^28 elements takes
    more than a minute), written past pytest's capture so that whoever watches the run sees
    that it is alive."""
    if _CAPTURE is not None:
        with _CAPTURE.global_and_fixture_disabled():
            print(f"\n[step] {msg}", file=sys.stderr, flush=True)
    else:
        print(f"[step] {msg}", file=sys.stderr, flush=True)


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
