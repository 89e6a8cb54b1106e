import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # A child test run may name another build of the library (the one with the large-launch
    # attention kernel pinned): the binding then loads that file instead of the shipped one.
    lib = os.environ.get("KVS_TEST_LIBRARY")
    if lib:
        from paper_2503_16525_amd import binding
        binding.LIB_PATH = lib


def _have_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """How much of the bf16 attention tolerance each parity case used (tests/attn_check.py)."""
    try:
        from attn_check import REPORT
    except Exception:
        return
    if REPORT:
        terminalreporter.section("attention tolerance records")
        for line in REPORT:
            terminalreporter.write_line(line)
