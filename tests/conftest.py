import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # Tests load the library that is already built; compile only if there is none.
    lib = os.path.join(ROOT, "paper_2605_04263_amd", "libpv.so")
    if not os.path.exists(lib):
        from paper_2605_04263_amd.build import build_library
        build_library(verbose=False)
