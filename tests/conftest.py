import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """Tests load what is built; only if nothing is built do they build it (hipcc cross-compiles
    gfx950 without a GPU).  The binding itself never builds: it fails loudly when the library is
    missing."""
    from paper_2512_05906_amd import build
    if not os.path.exists(build.LIB):
        build.build_library()
