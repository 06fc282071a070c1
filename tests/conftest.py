import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """How the bf16 output rule was used by the parity tests that ran (see parity_util.check_output)."""
    try:
        from parity_util import STATS
    except Exception:
        return
    if STATS["bf16_elements"]:
        terminalreporter.write_line(
            f"bf16 outputs compared: {STATS['bf16_elements']}; held to 2e-2: all below 8 in magnitude "
            f"(largest error {STATS['bf16_max_err_below_8']:.3e}); at or above 8: {STATS['bf16_wide']} "
            f"(largest error {STATS['bf16_wide_max_err']:.3e})")
