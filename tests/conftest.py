import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "expects_id_faults: the test feeds block ids outside the pool "
                                       "on purpose and checks the count itself")


@pytest.fixture(scope="session")
def device():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


@pytest.fixture(autouse=True)
def id_faults(request):
    """Every GPU test runs with the library's refused-id report switched on and must leave the
    counter at zero: no kernel met a block id outside its pool.  Tests that plant such ids are
    marked `expects_id_faults` and check the count themselves (through this fixture's tensor)."""
    if request.node.get_closest_marker("gpu") is None:
        yield None
        return
    import torch
    if not torch.cuda.is_available():
        yield None
        return
    from paper_2602_11530_amd import binding as pkv
    counter = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    torch.cuda.synchronize()
    pkv.pkv_set_id_fault_counter(counter)
    try:
        yield counter
        torch.cuda.synchronize()
        if request.node.get_closest_marker("expects_id_faults") is None:
            assert int(counter.item()) == 0, "a kernel refused a block id outside the pool"
    finally:
        pkv.pkv_set_id_fault_counter(None)
