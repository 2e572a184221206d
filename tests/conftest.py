import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_cfg():
    return dict(n_q_heads=4, n_kv_heads=2, head_dim=4, rms_eps=1e-6, rope_theta=1e4, pos_offset=0)
