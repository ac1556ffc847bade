import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built; they build it only if there is none
    from paper_2503_09304_amd.build import ensure_built
    ensure_built()


def pytest_collection_modifyitems(config, items):
    # GPU tests are selected with -m gpu; without a device they are skipped, never run on a
    # CPU fallback (there is none).
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    # The error figures the GPU parity tests measured (also for tests that passed, whose output pytest
    # does not show): one line per compared tensor.
    try:
        import gpu_util
    except Exception:  # pragma: no cover
        return
    if gpu_util.REPORT:
        terminalreporter.write_sep("-", "parity figures (GPU vs oracle)")
        for line in gpu_util.REPORT:
            terminalreporter.write_line(line)
