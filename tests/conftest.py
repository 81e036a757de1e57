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


@pytest.fixture(params=["plain", "ws", "ws_stream"])
def conv_entry(request):
    """Runs a convolution parity test once per entry point (see gpu_util.qconv2d); "ws_stream" also
    switches off the kernels specialised for 1x1 and 3x3 geometries, so that the streaming implicit
    GEMM over the workspace copies meets every geometry."""
    import gpu_util
    import paper_2103_14949_amd as hago
    gpu_util.CONV_ENTRY["name"] = "plain" if request.param == "plain" else "ws"
    if request.param == "ws_stream":
        hago.set_test_hook(hago.HOOK_GEMM_PATH, 2)
    yield request.param
    hago.set_test_hook(hago.HOOK_GEMM_PATH, 0)
    gpu_util.CONV_ENTRY["name"] = "plain"


@pytest.fixture
def stream_tile():
    """Forces a tile shape of the streaming dense kernel for the rest of a test."""
    import paper_2103_14949_amd as hago
    yield lambda tile: hago.set_test_hook(hago.HOOK_STREAM_TILE, tile)
    hago.set_test_hook(hago.HOOK_STREAM_TILE, -1)


@pytest.fixture
def gemm_path():
    """Forces the GEMM kernel family (1: general register-staged, 2: streaming without the kernels
    specialised for 1x1 and 3x3 convolutions) for the rest of a test."""
    import paper_2103_14949_amd as hago
    yield lambda path: hago.set_test_hook(hago.HOOK_GEMM_PATH, path)
    hago.set_test_hook(hago.HOOK_GEMM_PATH, 0)
