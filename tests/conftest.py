import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_stack():
    """Tiny fp32 three-model stack: weight blobs, prompt and config."""
    from paper_2510_12966_amd import synth

    cfg = synth.CONFIGS["tiny"]
    d, q, t, prompt = synth.build_stack(cfg)
    return cfg, d, q, t, prompt
