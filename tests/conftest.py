import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the library that is built; only when there is none do they build it (the binding itself
    never does: it fails loudly)."""
    lib = os.path.join(ROOT, "paper_2509_18085_amd", "libspiffy.so")
    if not os.path.exists(lib):
        from paper_2509_18085_amd import build
        build.build()


def pytest_terminal_summary(terminalreporter):
    """Reported, not gated: the counts the tests collected (see helpers.REPORT)."""
    import json
    helpers = sys.modules.get("helpers")
    records = getattr(helpers, "REPORT", []) if helpers else []
    if not records:
        return
    terminalreporter.section("reported counts (near-ties, excluded states, plain-oracle disagreements, error growth)")
    for r in records:
        terminalreporter.write_line(json.dumps(r))
    path = os.environ.get("SPIFFY_TEST_REPORT")
    if path:
        with open(path, "w") as f:
            for r in records:
                f.write(json.dumps(r) + "\n")
