import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Rows of whitespace-separated tokens; '#' starts a comment."""
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                rows.append(line.split())
    return rows


@pytest.fixture(scope="session")
def ref():
    from oracle import hago_ref
    hago_ref.build()
    hago_ref.lib()
    return hago_ref


@pytest.fixture(params=["plain", "ws"])
def conv_entry(request):
    """Runs a convolution parity test once per entry point (see gpu_util.qconv2d)."""
    import gpu_util
    gpu_util.CONV_ENTRY["name"] = request.param
    yield request.param
    gpu_util.CONV_ENTRY["name"] = "plain"


@pytest.fixture
def stream_tile():
    """Forces a tile shape of the streaming dense kernel for the rest of a test."""
    import paper_2103_14949_amd as hago
    yield lambda tile: hago.set_test_hook(hago.HOOK_STREAM_TILE, tile)
    hago.set_test_hook(hago.HOOK_STREAM_TILE, -1)


@pytest.fixture
def gemm_path():
    """Forces the GEMM kernel family (1: general register-staged, 2: streaming without the 1x1
    special cases) for the rest of a test."""
    import paper_2103_14949_amd as hago
    yield lambda path: hago.set_test_hook(hago.HOOK_GEMM_PATH, path)
    hago.set_test_hook(hago.HOOK_GEMM_PATH, 0)
