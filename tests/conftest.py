import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def small_cfg():
    from ded_inputs import ModelConfig
    return ModelConfig("pin-small", 2, 32, 4, 2, 8, 48, 50, dtype="fp32")


@pytest.fixture(scope="session")
def small_model(small_cfg):
    from ded_inputs import make_weights
    # std 0.3 keeps the soft-max far from uniform so that masking / ordering mistakes show up
    return make_weights(small_cfg, seed=3, gain_jitter=0.1, std=0.3)
