import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# a directory that holds another copy of the oracle package: the test that plants mistakes in such copies runs the
# pin tests against them in child processes
if os.environ.get("TR_ORACLE_PATH"):
    sys.path.insert(0, os.environ["TR_ORACLE_PATH"])
    import oracle  # noqa: F401  (bound now: pytest puts the repository root in front again when it imports the tests)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def _gpu_present():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    # GPU tests are selected with -m gpu on the GPU machine; without a device they are skipped
    # (never silently passed on a CPU fallback: there is none).
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)
