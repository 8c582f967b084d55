import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _redirect_binding_to_hostcheck_build():
    """QUARTET_HOSTCHECK_DIR (set by tests/test_sanitizers.py for its child run only): a directory holding a copy of the
    binding next to a host-only, sanitizer-instrumented build of the C ABI; tests that import the binding then drive that
    build instead of the HIP library."""
    d = os.environ.get("QUARTET_HOSTCHECK_DIR")
    if not d:
        return
    import importlib.util
    import paper_2505_14669_amd
    spec = importlib.util.spec_from_file_location("paper_2505_14669_amd.binding", os.path.join(d, "binding.py"))
    mod = importlib.util.module_from_spec(spec)
    sys.modules["paper_2505_14669_amd.binding"] = mod
    spec.loader.exec_module(mod)
    paper_2505_14669_amd.binding = mod


def pytest_configure(config):
    _redirect_binding_to_hostcheck_build()
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
