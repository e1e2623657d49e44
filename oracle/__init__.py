"""CPU oracle for the GPU library.  TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke
check and the benchmark's CPU-baseline leg; never by the served path."""
from . import ops, models  # noqa: F401
