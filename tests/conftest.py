import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import gemm_oracle
    gemm_oracle.lib()
    return gemm_oracle


@pytest.fixture(scope="session")
def level3_oracle():
    from oracle import gemm_oracle, level3_oracle
    gemm_oracle.lib()
    return level3_oracle
