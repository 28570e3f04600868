import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


_capture = None


def pytest_configure(config):
    global _capture
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    _capture = config.pluginmanager.getplugin("capturemanager")


def say(msg: str) -> None:
    """Progress line of a GPU test, printed past pytest's capture: it names the case before every GPU step, so a
    run that dies says where, and a long test is never silent."""
    if _capture is not None:
        with _capture.global_and_fixture_disabled():
            print(msg, flush=True)
    else:
        print(msg, flush=True)


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped, not failed, where no GPU is visible."""
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


GOLDEN = os.path.join(ROOT, "tests", "golden")


def read_golden_table(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            parts = line.split()
            rows[parts[0]] = [float(x) for x in parts[1:]]
    return rows
