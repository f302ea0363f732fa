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
    import oracle as _oracle
    _oracle.build()
    return _oracle


@pytest.fixture(autouse=True)
def _library_options_back_to_automatic():
    """fa_set_option is process-wide: whatever a test forced is undone after it."""
    yield
    import os as _os
    from paper_2410_16663_amd import binding
    if _os.path.exists(binding.LIB_PATH):
        import options
        options.reset_all()
