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
    from oracle import reference
    reference.build()
    return reference


@pytest.fixture
def knobs():
    """Sets the library's process-wide options (fp4_set_option) for one test and restores the defaults afterwards:
    knobs(variant=11, grid=2, sw_codec=1)."""
    from paper_2509_23202_amd import binding as fp4
    ids = {"variant": fp4.OPT_GEMM_VARIANT, "grid": fp4.OPT_GEMM_GRID, "sw_codec": fp4.OPT_SW_CODEC}

    def set_(**kw):
        for k, v in kw.items():
            fp4.set_option(ids[k], int(v))

    yield set_
    for o in ids.values():
        fp4.set_option(o, 0)
