import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the shared libraries are build products (not in the history): build them once if they are not there
    from paper_2602_11192_amd.build import ensure_built
    ensure_built()
    import oracle
    oracle.build()
