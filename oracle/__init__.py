"""CPU oracle for the verification step (NumPy float64 + integer Philox).

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this package.  It shares no code with
paper_2507_02659_amd (the HIP path) and neither imports the other.
"""
from . import philox, verify  # noqa: F401
