"""fp64 CPU oracles for fused attention and the fused RMS layer norm.  TEST INFRASTRUCTURE ONLY.

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
from .rmsnorm_oracle import rms_norm  # noqa: F401
from .kv_write_oracle import kv_cache_write  # noqa: F401
