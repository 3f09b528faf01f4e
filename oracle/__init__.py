"""CPU oracle for the TSVD forward map -- test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares nothing with the GPU library.
"""
from .tsvd_oracle import (  # noqa: F401
    build, forward, forward_columns, forward_layer, round_to_bf16, op_counts, acceleration,
    critical_rank, threads,
)
from . import transition  # noqa: F401  (Algorithms 1 and 2, Eq. 3, Theorem 1 in fp64 numpy)
from . import conv  # noqa: F401  (the four convolution forms through the dense kernel)
