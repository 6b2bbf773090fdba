"""CPU oracle (test infrastructure): ctypes front-end of oracle.c.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It never imports the HIP package and shares nothing with it.
"""
from .cpu_oracle import (
    OP_SUM, OP_MEAN, OP_GCN_SYM, OP_SAGE_GCN,
    build_oracle, compile_c, use_library, aggregate_fwd, aggregate_bwd, csr_indptr, transpose, plan, max_threads,
)

__all__ = [
    "OP_SUM", "OP_MEAN", "OP_GCN_SYM", "OP_SAGE_GCN", "build_oracle", "compile_c", "use_library", "aggregate_fwd", "aggregate_bwd",
    "csr_indptr", "transpose", "plan", "max_threads",
]
