import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box)")


@pytest.fixture(scope="session")
def cfg1_literal():
    from synth import get_config, make_workload
    return make_workload(get_config("cfg1"), device="cpu", noise="literal", keep_embeddings=4096)


@pytest.fixture(scope="session")
def cfg1_calibrated():
    from synth import get_config, make_workload
    return make_workload(get_config("cfg1"), device="cpu", noise="calibrated", keep_embeddings=4096)
