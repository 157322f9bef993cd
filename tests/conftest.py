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


@pytest.fixture
def tune():
    """tune(key, value): sets a launch-plan override of the library for the rest of the test."""
    from paper_2509_21081_amd import binding as T
    saved = []

    def _set(key, value):
        saved.append((key, T.typhoon_mla_set_tuning(key, value)))
    yield _set
    for key, old in reversed(saved):
        T.typhoon_mla_set_tuning(key, old)
