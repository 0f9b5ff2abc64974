import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle


@pytest.fixture(autouse=True)
def _library_options_back_to_default(request):
    """Tests switch kernels through ge_set_option; whatever a GPU test set is undone after it."""
    yield
    if request.node.get_closest_marker("gpu") is not None:
        from paper_2604_01489_amd import binding
        for name in ("force_config", "waves", "stage_k", "conv_halo"):
            binding.set_option(name, None)
