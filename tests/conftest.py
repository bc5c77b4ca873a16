import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "size_dispatch: the library picks the compress kernels by "
                            "shard size, as in bench.py (the tests at full workload sizes)")


@pytest.fixture(autouse=True)
def _kernel_choice_by_shard_size(request, monkeypatch):
    """The compress half at chunk 64 and 128 has two kernel choices and picks by shard size
    (DETO_SMALL_SHARD_TILES, include/detonation.h).  Test inputs are small, so left alone they
    would all run the small-shard choice: unless a test asks for the library's own choice
    (marker size_dispatch: the full-size workloads) or sets the variable itself
    (tests/test_gpu_small_shards.py runs both choices), the limit is 0 here and the kernels
    of large shards run.  DETO_TEST_SIZE_DISPATCH_EVERYWHERE=1 in the environment of a pytest run
    leaves the choice to the library in every test."""
    if os.environ.get("DETO_TEST_SIZE_DISPATCH_EVERYWHERE"):
        return      # a run of the whole suite on the library's own choice
    if request.node.get_closest_marker("size_dispatch") is None:
        monkeypatch.setenv("DETO_SMALL_SHARD_TILES", "0")
    else:
        monkeypatch.delenv("DETO_SMALL_SHARD_TILES", raising=False)


@pytest.fixture(scope="session")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")
