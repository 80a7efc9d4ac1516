import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def _qp_library():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2509_20214_amd as m
    m.load_library(build_if_missing=False)   # a missing library is an error, never a fallback
    return m


@pytest.fixture
def qp(_qp_library):
    """The binding, for GPU tests.  Tests steer kernels through qp_set_option; whatever a test set
    is back at its default for the next one."""
    _qp_library.qp_reset_options()
    yield _qp_library
    _qp_library.qp_reset_options()
