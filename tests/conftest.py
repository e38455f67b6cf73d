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


@pytest.fixture(scope="session", autouse=True)
def _kernel_path_from_env():
    """MLORA_TEST_KERNEL_PATH=<bits> runs the whole session with that test switch of
    include/mlora_testing.h set (kernel variants kept for comparison)."""
    kp = os.environ.get("MLORA_TEST_KERNEL_PATH")
    if kp:
        from paper_2312_02515_amd import binding
        binding.set_kernel_path(int(kp))
    yield
