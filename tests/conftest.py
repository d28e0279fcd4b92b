import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False

# the library's development switches must not leak into the tests: every test states the mode it checks
for _name in ("EINDECOMP_FUSE", "EINDECOMP_FUSE_AGG", "EINDECOMP_CONTRACT", "EINDECOMP_DMA_WAVES", "EINDECOMP_DMA_TILE"):
    if _name in os.environ and os.environ.get("EINDECOMP_TEST_KEEP_ENV") != "1":
        del os.environ[_name]
