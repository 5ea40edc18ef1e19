import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def device():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


@pytest.fixture(autouse=True)
def _fresh_tuning_cache():
    """fs_plan_tune records its winners per process and fs_plan_create reuses them: every test
    starts without any, so that default plans are the defaults whatever ran before."""
    try:
        from paper_1911_11576_amd import fs_tune_cache_clear
        fs_tune_cache_clear()
    except Exception:      # the tests of the oracle alone do not need the library
        pass
    yield
