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


@pytest.fixture(autouse=True)
def _no_tile_override_left_behind():
    """Tile overrides (conv_mcmk_force_tile / _gemm_tile) are process-wide: whatever a test forced is undone
    after it, pass or fail, so that no later test runs on a shape it did not ask for."""
    yield
    from paper_1704_04428_amd import binding
    if binding._lib is not None:
        binding.conv_mcmk_force_tile(-1)
        binding.conv_mcmk_force_gemm_tile(-1)
