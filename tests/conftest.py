import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def gpu():
    """The HIP binding with a CUDA(HIP) device; GPU tests only."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    import paper_2506_05413_amd as sr
    return sr


@pytest.fixture
def tune(gpu):
    """tune(knob, value): sets a tuning knob of the library for the duration of one test (all back to auto after)."""
    def set_knob(knob, value):
        gpu.sr_tune_set(knob, int(value))
    yield set_knob
    for knob in range(gpu.SR_TUNE_KNOBS):
        gpu.sr_tune_set(knob, gpu.SR_TUNE_AUTO)
