import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture
def tuning():
    """Sets launch-plan overrides of the library (kascade_tuning_set) and puts every knob back to 0 afterwards."""
    from paper_2512_16391_amd import binding

    def set_knob(knob, value):
        binding.kascade_tuning_set(knob, value)

    yield set_knob
    for knob in (binding.TUNE_DECODE_FAMILY, binding.TUNE_STREAM_CHUNK, binding.TUNE_GATHER_CHUNK, binding.TUNE_TOPK_PARTS):
        binding.kascade_tuning_set(knob, 0)
