import os
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU harness)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import grkan_oracle

    grkan_oracle.build()
    return grkan_oracle


@pytest.fixture(scope="session")
def oracle_np():
    from oracle import grkan_numpy

    return grkan_numpy
