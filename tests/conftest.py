import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_present() -> bool:
    try:
        import torch
        return bool(torch.cuda.is_available())
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


_T0 = None


def pytest_runtest_logstart(nodeid, location):
    """Names every test on stderr as it starts, with the seconds since the first one (a long
    GPU run that prints nothing for minutes looks hung to whoever is watching it)."""
    import time
    global _T0
    if _T0 is None:
        _T0 = time.time()
    sys.stderr.write("[test +%4.0fs] %s\n" % (time.time() - _T0, nodeid))
    sys.stderr.flush()
