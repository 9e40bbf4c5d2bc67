"""fp64 CPU oracle for fused attention.  TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this package; the product library never does.
"""
from .attn_oracle import (  # noqa: F401
    OracleProblem,
    attention,
    attention_rows,
    build,
    num_threads,
)
