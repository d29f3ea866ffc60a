import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--oracle-lib", default=None,
                     help="run the CPU pin tests against another build of oracle/tlin_oracle.c (mutation test only)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    lib = config.getoption("--oracle-lib")
    if lib:
        # a substitute oracle must never judge the GPU path
        markexpr = config.getoption("-m") or ""
        if "gpu" in markexpr and "not gpu" not in markexpr:
            raise pytest.UsageError("--oracle-lib is for the CPU pin tests and is refused when GPU tests are selected")
        import oracle
        oracle.use_library(lib)


@pytest.fixture(scope="session", autouse=True)
def _built_cpu_helpers():
    """The oracle and the input generator are small C files; build them if absent."""
    import oracle
    import tlin_inputs
    if not os.path.exists(oracle._LIB_PATH):
        oracle.build()
    if not os.path.exists(tlin_inputs._LIB_PATH):
        tlin_inputs.build()
