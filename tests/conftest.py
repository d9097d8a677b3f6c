import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")
    san = os.environ.get("TBE_SANITIZED_LIBS")
    if san:  # tests/sanitize_cpu_side.py: the oracle and the host-only solver built with ASan + UBSan
        import ctypes
        import oracle
        from paper_2305_01515_amd import placement
        oracle._LIB = os.path.join(san, "libtbe_oracle_san.so")
        oracle.build = lambda force=False: oracle._LIB
        solver = ctypes.CDLL(os.path.join(san, "libtbe_place_san.so"))
        placement._solver_library = lambda: solver


@pytest.fixture(autouse=True, scope="module")
def _release_cached_memory():
    """GPU test modules pin several GB of host memory each (the backing tiers).  torch keeps freed
    pinned blocks in a cache, and the box refuses to pin more than about 64 GiB in total, so the
    caches are emptied after every module: a later module with big tables must not fail on what
    an earlier one left behind."""
    yield
    import gc
    import torch
    if torch.cuda.is_available():
        gc.collect()
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        torch._C._host_emptyCache()
