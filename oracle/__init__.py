"""CPU oracle for online resharding of mixed-parallel training state.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its
Python binding) may import this package; only the tests, the smoke check and
the CPU-baseline leg of the benchmark do.  It shares no code with the HIP path.
"""
from .reshard_oracle import *  # noqa: F401,F403
