import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")


@pytest.fixture(scope="session")
def tiny_cfg():
    """A two-level shape small enough for pure-Python brute force."""
    from paper_2505_23317_amd import synth
    return synth.Config("tiny", 2, 64, 64, (16, 8), 16, 2, 2, 32, "f32",
                        frac_lo=0.0, frac_hi=0.2, box_rule="fraction",
                        side_lo=8, side_hi=24)
