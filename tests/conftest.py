import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_finish(session):
    """The full-size parity tests fan the oracle out over CPU-only worker processes.  They are forked here,
    once collection is done and before any test (or fixture) makes the process's first GPU call; counting
    devices does not initialise the GPU."""
    if not any(item.get_closest_marker("gpu") for item in session.items):
        return
    try:
        import torch
        if torch.cuda.device_count() < 1:
            return
    except Exception:
        return
    from oracle import pool as oracle_pool
    oracle_pool.start()


def pytest_sessionfinish(session, exitstatus):
    from oracle import pool as oracle_pool
    oracle_pool.stop()


def has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


@pytest.fixture(scope="session")
def gpu_device():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


@pytest.fixture(scope="session")
def oracle_workers(gpu_device):
    from oracle import pool as oracle_pool
    if not oracle_pool.started():
        pytest.skip("oracle workers were not started (no GPU test was collected)")
    return oracle_pool
