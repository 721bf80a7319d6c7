import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for _p in (ROOT, os.path.dirname(os.path.abspath(__file__))):
    if _p not in sys.path:
        sys.path.insert(0, _p)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    import pg_progress as progress
    progress.set_config(config)
    from paper_2512_15347_amd.build import ensure_built
    ensure_built()                                   # compiles only when no library has been built yet


@pytest.fixture(scope="session")
def lib():
    """The HIP library through its Python binding; GPU tests fail loudly without it."""
    from paper_2512_15347_amd import binding
    return binding
