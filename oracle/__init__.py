"""CPU oracle for the multi-rail allreduce arithmetic (test infrastructure).

Only tests, the smoke check and the CPU-baseline leg of the benchmark may
import this package.  It never imports the GPU package and the GPU package
never imports it.
"""
from .nz_oracle import *  # noqa: F401,F403
