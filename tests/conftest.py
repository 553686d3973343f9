import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def small_layers():
    """A few small rectangular layers shared by the CPU tests (built once)."""
    from paper_2504_19449_amd import synth
    out = {}
    for name, (d_in, d_out, r, dt) in {
        "wide_f16": (96, 40, 12, synth.F16),
        "tall_bf16": (48, 112, 16, synth.BF16),
        "square_f16": (64, 64, 64, synth.F16),
    }.items():
        out[name] = synth.make_layer(d_in, d_out, r, dt, config=90, linear=len(out))
    return out
