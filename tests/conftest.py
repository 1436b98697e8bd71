import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The tests load the library that is built.  It is built here (hipcc cross-compiles without a GPU) when there is
    # none, or - on a machine without a GPU, where the sources are edited - when a source or header is newer than it,
    # so that no test runs against code that was never compiled.  A machine with a GPU receives the tree as a copy
    # (file times are those of the copy): it runs the library it was sent.
    pkg = os.path.join(ROOT, "paper_2503_02508_amd")
    lib = os.path.join(pkg, "libqc.so")
    srcs = [os.path.join(d, f) for d in (os.path.join(pkg, "csrc"), os.path.join(ROOT, "include"))
            for f in os.listdir(d) if f.endswith((".hip", ".h"))]
    stale = not os.path.exists(lib) or (not _have_gpu() and any(os.path.getmtime(f) > os.path.getmtime(lib) for f in srcs))
    if stale:
        import shutil
        if shutil.which("hipcc") or os.path.exists("/opt/rocm/bin/hipcc"):
            import importlib.util
            spec = importlib.util.spec_from_file_location("qc_build", os.path.join(pkg, "build.py"))
            b = importlib.util.module_from_spec(spec)
            spec.loader.exec_module(b)
            b.build()
        elif os.path.exists(lib):
            raise pytest.UsageError("libqc.so is older than its sources and there is no hipcc to rebuild it")


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
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)
