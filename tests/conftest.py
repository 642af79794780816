import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--sanitizers", action="store_true",
                     help="also run the sanitizer leg (tests/test_sanitizers.py): the oracle and the host code of the "
                          "HIP library rebuilt with AddressSanitizer + UndefinedBehaviorSanitizer, CPU tests only")
    parser.addoption("--bsr-libs", default=None,
                     help="load libbsr_oracle_*.so from this directory (what the sanitizer leg starts its child process with)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    libs = config.getoption("--bsr-libs")
    if libs:
        import oracle.binding as ob
        ob._lib_path = lambda prec: os.path.join(libs, f"libbsr_oracle_{prec}.so")


@pytest.fixture(scope="session")
def orc64():
    from oracle import Oracle
    return Oracle("f64")


@pytest.fixture(scope="session")
def orc32():
    from oracle import Oracle
    return Oracle("f32")
