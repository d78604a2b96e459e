import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_generate_tests(metafunc):
    """Every GPU test runs twice: with fp32 and with bf16 summary vectors (the library's storage switch; the oracle
    follows through helpers.geom_of).  A module whose tests never touch the summaries opts out with
    ``SUMMARY_DTYPE_SWEEP = False``."""
    if metafunc.definition.get_closest_marker("gpu") is None:
        return
    if getattr(metafunc.module, "SUMMARY_DTYPE_SWEEP", True):
        metafunc.parametrize("_summary_dtype", [0, 1], ids=["f32", "bf16"], indirect=True)


@pytest.fixture(autouse=True)
def _summary_dtype(request):
    import helpers
    helpers.SUMMARY_DTYPE = getattr(request, "param", 0)
    yield helpers.SUMMARY_DTYPE
    helpers.SUMMARY_DTYPE = 0
