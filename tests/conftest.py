import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no device is visible.
    try:
        import torch
        have = torch.cuda.is_available()
    except Exception:
        have = False
    if have:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture(autouse=True)
def _library_options_back_to_default(request):
    """Tests steer the library through spqr_set_option (process-wide): every test leaves the defaults behind."""
    yield
    if "gpu" in request.keywords:
        import paper_2306_03078_amd as P
        for opt in (P.SPQR_OPT_BATCH_PATH, P.SPQR_OPT_FORCE_GENERIC, P.SPQR_OPT_BATCH_STEPS, P.SPQR_OPT_DENSE_ROWS, P.SPQR_OPT_GEMV_PLAN):
            P.spqr_set_option(opt, 0)
