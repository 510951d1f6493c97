import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # Tests load the library that is already built; compile only if there is none, or if a source
    # is newer than it (a stale binary would be tested against the wrong code).
    from paper_2605_04263_amd import build
    if build.library_is_stale():
        build.build_library(verbose=False)
