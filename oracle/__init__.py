"""Plain fp64 CPU oracle for the PackCache hot path.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product:
only the tests, the smoke check and the CPU-baseline leg of the benchmark may
import it.  It shares no code with the HIP library and never imports it.
"""
from .packcache_oracle import *  # noqa: F401,F403
