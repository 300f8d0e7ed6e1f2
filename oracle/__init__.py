"""CPU reference for the DAT worker step (test infrastructure, not the product).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It never imports the GPU package and shares no code with it.
"""
from .cpu import *  # noqa: F401,F403
