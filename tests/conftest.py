import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The binding refuses to run without a built library; the test session builds it once if
    # nothing is there (a fresh checkout), and otherwise loads what is built.
    from paper_2512_10411_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2512_10411_amd.build import build_library
        build_library()
