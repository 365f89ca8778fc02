"""pytest configuration: marker registration, import path, and a built library for the host-side tests."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_sessionstart(session):
    # A fresh checkout has no libhgemm.so (built artefacts are not committed).  The host-side tests
    # load it, so compile it once if it is missing; an existing library is used as it is.
    from paper_2512_02551_amd import build

    if not os.path.exists(build.LIB):
        build.build(force=True)
