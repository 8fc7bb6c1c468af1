import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped (not failed) when no device is present and the run did not ask
    for them explicitly with -m gpu."""
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """The GPU parity tests record every measured error; leave the table behind."""
    mod = sys.modules.get("tests.gpu_util")
    if mod is not None:
        path = mod.write_records()
        if path:
            print(f"\n[parity] {len(mod.RECORDS)} measured errors written to {path}")
