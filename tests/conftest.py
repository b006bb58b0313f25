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


@pytest.fixture(params=["default flow", "large-input kernels"])
def flow(request):
    """Hard curves of small and mid-sized float grids without a range (up to 2^27 vertices in images,
    2^25 in volumes, up to 4096 items, up to 4096 bins) take two- or three-launch flows of their own.
    A test that asks for this fixture runs twice: as a caller gets it, and with those flows switched
    off, so that the five-launch flow of the large inputs -- shared lists, the second sweep in
    reserve, the generic kernels -- still meets the same small and ragged shapes."""
    from paper_2510_20271_amd import api
    prev = api.ecc_debug_force(0 if request.param == "default flow" else api.ECC_FORCE_NO_SMALL)
    yield request.param
    api.ecc_debug_force(prev)
