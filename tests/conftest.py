"""Shared pytest configuration: the `gpu` marker and import paths."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--oracle-lib", default=None,
                     help="run the oracle pins against this shared library instead of the built oracle "
                          "(used only by tests/test_oracle_mutations.py for its child runs)")


    parser.addoption("--pdelta-lib", default=None,
                     help="load the C-ABI library from this path instead of the in-tree libpdelta.so "
                          "(used only by tests/test_sanitizers.py for its child run of the host-side tests)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    path = config.getoption("--oracle-lib")
    if path:
        from oracle import pdelta_oracle
        pdelta_oracle.use_library(path)
    path = config.getoption("--pdelta-lib")
    if path:
        from paper_2512_19720_amd import binding
        binding._LIB_PATH = path


def pytest_sessionstart(session):
    """Load what is built; build only if nothing is (hipcc cross-compiles without a GPU)."""
    lib = os.path.join(ROOT, "paper_2512_19720_amd", "libpdelta.so")
    if not os.path.exists(lib):
        from paper_2512_19720_amd import build as pdelta_build
        pdelta_build.build_library()
