import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def dims():
    from paper_2211_13939_amd import synth
    return dict(synth.DIMS)


@pytest.fixture(scope="session")
def weights_fp32():
    from paper_2211_13939_amd import synth
    return synth.make_weights()


@pytest.fixture(scope="session")
def weights_bf16():
    from paper_2211_13939_amd import synth
    return synth.make_weights(bf16=True)
