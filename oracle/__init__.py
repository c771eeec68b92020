"""CPU oracle for the AGoQ quantization hot path -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import this package.  It never imports the GPU package.
"""
from .ref import *  # noqa: F401,F403
