import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the library that is built; only when none is there do they build it once
    (hipcc cross-compiles gfx950 without a GPU).  The binding itself never builds and never falls back."""
    from paper_2512_24086_amd import rf2
    if not os.path.exists(rf2.LIB_PATH):
        from paper_2512_24086_amd.build import build
        build(verbose=False)
