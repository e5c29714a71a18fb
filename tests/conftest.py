import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as o

    o.build()
    return o


def pytest_terminal_summary(terminalreporter):
    """Lists the worst error of every kind of comparison the parity tests made (bf16 bound: 2e-2 absolute)."""
    try:
        from tests.util import ERRORS
    except Exception:
        return
    if not ERRORS:
        return
    worst = {}
    for what, e, mx in ERRORS:
        kind = " ".join(w for w in what.split() if not w.isdigit() and w != "head")
        if kind not in worst or e > worst[kind][0]:
            worst[kind] = (e, mx)
    if os.environ.get("MUSE_TEST_ALL_ERRORS"):   # every comparison, not only the worst of its kind
        for what, e, mx in ERRORS:
            terminalreporter.write_line(f"  each: {what:44s} {e:.3e}  {mx:.3g}")
    terminalreporter.write_line("parity errors (max abs err, max|want|), worst per comparison kind:")
    for kind in sorted(worst):
        terminalreporter.write_line(f"  {kind:40s} {worst[kind][0]:.3e}  {worst[kind][1]:.3g}")
