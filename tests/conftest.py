import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """Report the measured share of new cache entries that matched the oracle bit for bit."""
    try:
        from gpu_common import KV_BIT_EQUAL
    except Exception:
        return
    if KV_BIT_EQUAL:
        terminalreporter.write_line(f"new layer-0 K/V entries bit-equal to the oracle: min {min(KV_BIT_EQUAL):.4f} "
                                    f"mean {sum(KV_BIT_EQUAL) / len(KV_BIT_EQUAL):.4f} over {len(KV_BIT_EQUAL)} checks")
