"""CPU oracle (test infrastructure): ctypes front-end of oracle.c, ap_oracle.c and layer_oracle.c.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It never imports the HIP package and shares nothing with it.
"""
from .cpu_oracle import (
    OP_SUM, OP_MEAN, OP_GCN_SYM, OP_SAGE_GCN,
    build_oracle, compile_c, use_library, aggregate_fwd, aggregate_bwd, csr_indptr, transpose, plan, blocked_layout, max_threads,
    BIN_ADD, BIN_SUB, BIN_MUL, BIN_DIV, BIN_COPY_LHS, BIN_COPY_RHS, RED_SUM, RED_MAX, RED_MIN, ap_fwd, ap_bwd,
    matmul, sage_layer_fwd, sage_layer_bwd, SOURCES,
)

__all__ = [
    "OP_SUM", "OP_MEAN", "OP_GCN_SYM", "OP_SAGE_GCN", "build_oracle", "compile_c", "use_library", "aggregate_fwd", "aggregate_bwd",
    "csr_indptr", "transpose", "plan", "blocked_layout", "max_threads",
    "BIN_ADD", "BIN_SUB", "BIN_MUL", "BIN_DIV", "BIN_COPY_LHS", "BIN_COPY_RHS", "RED_SUM", "RED_MAX", "RED_MIN",
    "ap_fwd", "ap_bwd", "matmul", "sage_layer_fwd", "sage_layer_bwd", "SOURCES",
]
