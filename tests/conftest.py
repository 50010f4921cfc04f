import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _build_if_nothing_is_built():
    """A fresh checkout has no binaries: build them once (hipcc cross-compiles without a GPU).  What is built is
    used as it is; after a change to a source, build again by hand."""
    needed = [os.path.join(ROOT, "paper_2512_22560_amd", "librollattn.so"), os.path.join(ROOT, "tests", "libc_abi_client.so"),
              os.path.join(ROOT, "oracle", "libbrute_attn.so")]
    if all(os.path.exists(p) for p in needed):
        return
    import __graft_entry__
    __graft_entry__.build()


def pytest_configure(config):
    _build_if_nothing_is_built()
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library on cuda:0)")


def pytest_collection_modifyitems(config, items):
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
