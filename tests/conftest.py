import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--sweep-scale", type=int, default=1,
                     help="multiplies the number of seeds of the random sweeps in tests/test_gpu_sweep.py")


def pytest_generate_tests(metafunc):
    # a test that takes `sweep_seed` runs once per seed: two seeds by default, 2 * --sweep-scale on request
    if "sweep_seed" in metafunc.fixturenames:
        metafunc.parametrize("sweep_seed", list(range(2 * max(1, metafunc.config.getoption("--sweep-scale")))))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def dq():
    """The Python binding over the C-ABI library; fails loudly if the library is not built."""
    import paper_2405_12591_amd as lib
    return lib
