import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built; only a tree without one builds it here
    import __graft_entry__
    __graft_entry__.ensure_built()


def pytest_report_header(config):
    """The library under test: the hash of the sources it was compiled from (and of the tree's)."""
    from paper_2508_19740_amd import build as hip_build
    return f"libspotlight build id {hip_build.built_id()} (sources in the tree: {hip_build.source_id()})"


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, on a machine without a GPU when selected by accident.
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_runtest_logstart(nodeid, location):
    """A GPU run names each test, flushed, before it starts: the full-size tests take a minute
    each, and when a kernel faults the last line says which case it was."""
    item_is_gpu = "test_gpu_" in nodeid
    if not item_is_gpu:
        return
    sys.__stderr__.write(f"[gpu test] {nodeid}\n")
    sys.__stderr__.flush()
