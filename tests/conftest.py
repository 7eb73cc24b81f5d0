import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_np():
    """Config-1 module 0 as fp64 numpy arrays."""
    import numpy as np
    from paper_2510_03246_amd import inputs

    cfg = inputs.CONFIGS["tiny"]
    m = inputs.make_ffn_module(cfg, layer=0, seed=0)
    return cfg, {k: v.double().numpy() for k, v in m.items()}
