import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped (not failed) on a machine without a GPU unless
    they were asked for with -m gpu; then a missing GPU or a missing HIP
    library is an error raised by the tests themselves."""
    markexpr = config.getoption("-m") or ""
    if "gpu" in markexpr and "not gpu" not in markexpr:
        return
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU here (GPU tests run with -m gpu on the GPU box)")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """A session that ran on the debug build of the library (SKETCH_LINEAR_LIB names it) fails if any of its
    kernels counted a range-assert violation."""
    if "debug" not in os.path.basename(os.environ.get("SKETCH_LINEAR_LIB", "")):
        return
    import paper_2506_17255_amd as skl
    try:
        import torch
        if torch.cuda.is_available():
            torch.cuda.synchronize()
        count, first = skl.sketch_linear_debug_violations()
    except skl.SketchLinearError as e:
        print(f"\nrange asserts: {e}")
        session.exitstatus = 1
        return
    print(f"\nrange asserts of the debug build: {count} violation(s)" + (f", first {first}" if count else ""))
    if count:
        session.exitstatus = 1
