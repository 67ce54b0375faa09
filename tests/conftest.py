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


def read_golden(name: str) -> dict:
    """Parse a 'key value' text fixture; '#' starts a comment."""
    out = {}
    with open(golden_path(name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split(None, 1)
            out[k] = v.strip()
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden


@pytest.fixture(scope="session", autouse=True)
def _built_library():
    """Tests load the library that is built in-tree; it is rebuilt when it is absent or older than a source
    (where a compiler is at hand: the GPU machine runs what was built before the run)."""
    import shutil
    from paper_2203_00091_amd import build as b
    have_hipcc = shutil.which(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")) is not None
    if not os.path.exists(b.LIB) or (b.is_stale() and have_hipcc and not os.environ.get("DFSS_NO_REBUILD")):
        b.build()
    yield
