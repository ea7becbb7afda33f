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
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_report_header(config):
    """Which library binary the tests run against, and the digest of the sources it was built from."""
    try:
        from paper_2104_14129_amd import binding as B
        return f"libactq: {B.LIB_PATH} (source digest {B.source_hash()}, version {B.version()})"
    except Exception as exc:     # reported, never hidden: the ABI tests fail on their own
        return f"libactq: not loadable ({type(exc).__name__}: {exc})"
