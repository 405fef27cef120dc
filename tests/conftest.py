import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The tests load the library that is built; only when there is none (a fresh checkout) is it built here.
    from paper_2408_12526_amd import build as hip_build
    if not os.path.exists(hip_build.LIB):
        hip_build.build(verbose=False)


@pytest.fixture(scope="session")
def oracle64():
    from oracle.sp_oracle import Oracle
    return Oracle("f64")


@pytest.fixture(scope="session")
def oracle32():
    from oracle.sp_oracle import Oracle
    return Oracle("f32")
