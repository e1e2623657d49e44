import os
import sys

import pytest

# More hardware queues than HIP's default of 4: the co-location tests use five streams (two
# compute, two copy, the null stream) and two streams that share a hardware queue serialise.
os.environ.setdefault("GPU_MAX_HW_QUEUES", "8")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
