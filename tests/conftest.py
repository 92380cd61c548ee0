import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle

    _oracle.build()
    return _oracle


@pytest.fixture(scope="session", autouse=True)
def _final_path_from_env():
    """TLI_FINAL_PATH=1|2 runs the whole suite with one form of tli_verify's extra-token step forced (see
    tli_tune_final_path); unset, the library chooses by shape."""
    v = os.environ.get("TLI_FINAL_PATH")
    if v:
        from paper_2502_05202_amd import binding

        binding.tli_tune_final_path(int(v))
    yield
