"""CPU oracle for the LEANN search hot path (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with paper_2506_08276_amd.
"""
from .oracle import *  # noqa: F401,F403
