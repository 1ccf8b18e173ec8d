import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def repo_root():
    return ROOT


@pytest.fixture(scope="session")
def gpu():
    """Device and ONE pair of streams for the whole session. HIP maps streams round-robin onto a few
    hardware queues (GPU_MAX_HW_QUEUES, 4 here): if every test module made its own pair, a compute and
    a copy stream would end up on the same queue, and on the stream backend the flag writes of a
    resident run would then sit behind the kernel that waits for them (its bounded wait turns that
    into FICCO_ERR_TIMEOUT)."""
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2512_10236_amd as ficco
    torch.cuda.set_device(0)
    ficco.load()                      # fails loudly if the HIP library is missing
    return dict(dev=torch.device("cuda:0"), cs=torch.cuda.Stream(), xs=torch.cuda.Stream())
