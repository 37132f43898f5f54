import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped, not failed, where no GPU is present and -m gpu was not asked."""
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True)
def _library_decides_again_after_each_test():
    """Tests force code paths through grass_set_test_option; whatever a test set is cleared
    when it ends, so that no test depends on the one before it."""
    yield
    from paper_2406_17660_amd import grass
    if grass._lib is not None:
        for option in (grass.TEST_GEMM_TILE, grass.TEST_FUSED_STATS, grass.TEST_PACK_MXT,
                       grass.TEST_NO_PAIRS, grass.TEST_MAX_K_SLICES, grass.TEST_NO_NARROW_GATHER):
            grass.set_test_option(option, 0)
