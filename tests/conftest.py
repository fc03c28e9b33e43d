import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture
def pinned_gemm():
    """Pins the GEMM kernel variant for one test (quota_set_gemm_variant) and restores the automatic
    choice afterwards."""
    from paper_2604_17320_amd import binding
    yield binding.quota_set_gemm_variant
    binding.quota_set_gemm_variant(-1)
