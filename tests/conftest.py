import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden_path(name: str) -> str:
    return os.path.join(ROOT, "tests", "golden", name)


@pytest.fixture(scope="session")
def golden():
    return golden_path


@pytest.fixture(scope="session")
def wq():
    """The ctypes binding; builds libwq.so first only if no built library exists."""
    from paper_2412_19867_amd import wq as binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2412_19867_amd import build
        build.build_library()
    binding.lib()
    return binding
