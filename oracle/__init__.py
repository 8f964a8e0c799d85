"""CPU oracle for the HSD verification hot path (test infrastructure only).

Nothing in the product path (the HIP library and its Python binding) may import this package;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.
"""
from .hsd_oracle import *  # noqa: F401,F403
