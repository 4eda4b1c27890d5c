import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(autouse=True)
def _kernel_choice_back_to_default():
    """Tests force kernel choices through apnn_debug_force; none of them leaks into the next test."""
    yield
    from paper_2106_12169_amd import binding
    if binding._lib is not None:
        binding.apnn_debug_reset()
