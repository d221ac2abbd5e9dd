import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def toy_shape():
    from paper_2404_18911_amd import inputs
    return inputs.SHAPES["toy"]


@pytest.fixture(scope="session")
def toy_weights(toy_shape):
    from paper_2404_18911_amd import inputs
    return inputs.gen_weights(toy_shape, seed=1, alpha=0.1)
