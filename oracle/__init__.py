"""CPU oracle for the ESSA hot path. TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package. It shares no code with the HIP library and never imports it.
"""
from .essa_oracle import *  # noqa: F401,F403
from .essa_optimizers import *  # noqa: F401,F403,E402
