"""CPU oracle for the exact-GP hot path. TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may
import this package. The product path (paper_1903_08114_amd) never does, and
this package never imports the product path. See oracle/gp_dense.py.
"""
from .gp_dense import *  # noqa: F401,F403
