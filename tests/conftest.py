import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return ROOT / "tests" / "golden"


@pytest.fixture(scope="session")
def amlib():
    """The built C-ABI library through its binding; built here only when nothing has been built yet."""
    from paper_2601_22442_amd.build import LIB, build_library
    if not LIB.exists():
        build_library(force=True)
    import paper_2601_22442_amd as am
    return am
