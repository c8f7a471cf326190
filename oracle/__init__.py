"""CPU oracles (NumPy float64 + integer Philox): the verification step (verify, philox), the n-gram cache's life
cycle (ngram_cache), the hybrid distillation loss (distill) and the adaptive-drafting rule (adaptive).

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this package.  It shares no code with
paper_2507_02659_amd (the HIP path) and neither imports the other.
"""
from . import philox, verify  # noqa: F401
