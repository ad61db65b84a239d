import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the in-tree libraries; they are compiled here only if nothing has been built yet
    (hipcc cross-compiles for gfx950 without a GPU)."""
    from paper_2409_20476_amd import build
    build.ensure_built()
