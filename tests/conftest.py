import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def grid16():
    from paper_2501_19392_amd import synth
    return synth.lloyd_codebook(16)


@pytest.fixture(scope="session")
def grid64():
    from paper_2501_19392_amd import synth
    return synth.lloyd_codebook(64)
