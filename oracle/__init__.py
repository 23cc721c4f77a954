"""CPU oracle for the CALS hot path.  TEST INFRASTRUCTURE: imported only by tests/, by the smoke
check and by the benchmark's CPU-baseline leg; never by the product package."""
from .oracle import *  # noqa: F401,F403
