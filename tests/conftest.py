import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are selected with -m gpu; without a device they are skipped, never silently passed.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    # PTENC_ERROR_LOG=<file>: the largest errors every parity comparison of this session observed, as JSON
    path = os.environ.get("PTENC_ERROR_LOG")
    if not path:
        return
    import json
    from tests import helpers
    with open(path, "w") as fh:
        json.dump({k: {"max_abs": a, "max_row_rel": r} for k, (a, r) in sorted(helpers.OBSERVED.items())}, fh, indent=1)
