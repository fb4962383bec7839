import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the library that is built; a tree in which nothing is built yet gets built once, here (the binding
    itself never builds: it raises if the library is missing)."""
    from paper_1911_11377_amd import build as lib_build

    if not os.path.exists(lib_build.LIB):
        lib_build.build(force=True)
