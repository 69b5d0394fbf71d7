"""CPU oracle for multi-Bulyan (test infrastructure only).

Only tests, the smoke check and the CPU-baseline leg of the benchmark may
import this package.  It shares nothing with the GPU library.
"""
from .mbulyan_oracle import *  # noqa: F401,F403
