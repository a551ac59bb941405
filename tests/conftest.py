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


def pytest_collection_finish(session):
    """The oracle runs of the large configurations take minutes: when their GPU tests are among the
    selected ones, start them now, in background threads, so that they overlap with the tests
    that run first."""
    wanted = sorted({item.callspec.params["name"] for item in session.items
                     if "test_gpu_whole_configs" in item.nodeid and hasattr(item, "callspec")
                     and "name" in item.callspec.params})
    if wanted and not session.config.option.collectonly:
        from tests import whole_refs
        whole_refs.start(wanted)
