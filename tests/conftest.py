import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu_device():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


@pytest.fixture(params=["by-size", "cache-as-is", "transposed-copy"])
def v_source(request):
    """Where the pipelined attention kernel (head_dim 128, bf16) takes the values from: the
    library's own choice by problem size, always the cache as it is (transposed on the way
    out of LDS), or always a transposed copy made by a pre-pass.  The library reads the
    variable at every call; other geometries ignore it."""
    old = os.environ.get("PKV_ATTN_VT")
    if request.param == "by-size":
        os.environ.pop("PKV_ATTN_VT", None)
    else:
        os.environ["PKV_ATTN_VT"] = "0" if request.param == "cache-as-is" else "1"
    yield request.param
    if old is None:
        os.environ.pop("PKV_ATTN_VT", None)
    else:
        os.environ["PKV_ATTN_VT"] = old
