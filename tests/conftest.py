import os
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library through its C ABI)")


@pytest.fixture(scope="session")
def ss():
    """The Python binding over the C-ABI library; GPU tests only."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_00288_amd as pkg
    return pkg


@pytest.fixture
def force_tile(ss):
    """Forces the workgroup tile of the convolution kernels through the library's test hook (include/ss_debug.h);
    the library's own choice is restored afterwards.  `None` = the library chooses."""
    def setter(tid):
        ss.ss_debug_force_tile(-1 if tid is None else int(tid))
    yield setter
    ss.ss_debug_force_tile(-1)


@pytest.fixture
def limit_blocks(ss):
    """Caps the workgroups of the resident-grid kernels through the library's test hook; removed afterwards."""
    def setter(n):
        ss.ss_debug_limit_blocks(0 if n is None else int(n))
    yield setter
    ss.ss_debug_limit_blocks(0)


@pytest.fixture
def force_split(ss):
    """Forces the number of workgroups per output tile (split reduction) through the library's test hook."""
    def setter(n):
        ss.ss_debug_force_split(0 if n is None else int(n))
    yield setter
    ss.ss_debug_force_split(0)
