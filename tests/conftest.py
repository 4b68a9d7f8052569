import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The built libraries are not under version control.  A fresh checkout
    builds them once before the first test needs them (hipcc cross-compiles for
    gfx950 without a GPU; the oracle needs only gcc)."""
    import shutil
    lib = os.path.join(ROOT, "paper_2308_15164_amd", "libabs_sgd.so")
    if not os.path.exists(lib) and shutil.which("hipcc"):
        from paper_2308_15164_amd.build import build_library
        from bench_probe.build import build_probe
        build_library(force=True)
        build_probe()
