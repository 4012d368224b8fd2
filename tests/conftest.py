import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def lib():
    """The GPU library through its Python binding; fails loudly if it is not built."""
    import paper_2302_13053_amd as retexo
    retexo.binding.load()
    return retexo


@pytest.fixture(params=["few_rows", "row_blocks"])
def transform_family(request):
    """Runs a test twice: with the dense transform's few-rows kernel (what matrices of test size take) and with
    it switched off, i.e. on the 128-row block kernels that large matrices take."""
    from paper_2302_13053_amd import binding as B
    B.load()
    B.check(B.retexo_set_option("transform_few_blocks", 128 if request.param == "few_rows" else 0), "set_option")
    yield request.param
    B.check(B.retexo_set_option("transform_few_blocks", 128), "set_option")
