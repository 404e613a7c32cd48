import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
TESTS = os.path.dirname(os.path.abspath(__file__))
if TESTS not in sys.path:
    sys.path.insert(0, TESTS)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built in-tree; only when there is none do they build it (hipcc cross-compiles
    # for gfx950 without a GPU)
    lib = os.path.join(ROOT, "paper_2402_05109_amd", "libhydra.so")
    if not os.path.exists(lib):
        from paper_2402_05109_amd.build import build_library
        build_library(verbose=False)
