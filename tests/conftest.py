import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def to_np32(t):
    """torch tensor (f32 or bf16) -> float32 numpy; bf16 widens exactly."""
    return t.detach().to("cpu").float().numpy()


@pytest.fixture(scope="session")
def oracle():
    from oracle import hexa_oracle
    hexa_oracle.build()
    return hexa_oracle
