"""CPU oracle (test infrastructure).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It never imports the HIP path.
"""
from .oracle import *  # noqa: F401,F403
