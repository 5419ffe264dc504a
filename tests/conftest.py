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
    """The built C-ABI library through its binding.  Built here only when nothing has been built yet;
    a library that does not carry the digest of the source files beside it is refused, not rebuilt."""
    from paper_2601_22442_amd.build import LIB, build_library, check_library_is_current
    if not LIB.exists():
        build_library(force=True)
    import paper_2601_22442_amd as am
    check_library_is_current(am.version())
    return am
