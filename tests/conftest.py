import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The libraries are built in-tree beforehand; only if nothing is built at all (a fresh checkout)
    # are they compiled here, once.
    from paper_2605_11215_amd import build
    if not (os.path.exists(build.LIB) and os.path.exists(build.SYNTH_LIB) and os.path.exists(build.EXAMPLE)):
        build.build_all()


def pytest_collection_modifyitems(config, items):
    """GPU tests must never be silently skipped on a GPU machine and never run on a CPU machine."""
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
