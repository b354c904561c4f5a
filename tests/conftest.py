"""pytest configuration: markers, import path, and the oracle build."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")


@pytest.fixture(scope="session", autouse=True)
def _built():
    """Load what is built; build only what is missing (the oracle with gcc, the HIP library with
    hipcc -- cross-compiling needs no GPU)."""
    import oracle
    oracle.build()
    from paper_2104_02184_amd import binding, build as hip_build
    if not os.path.exists(binding.library_path()):
        hip_build.build(force=True)
    yield
