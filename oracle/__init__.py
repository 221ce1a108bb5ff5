"""CPU oracle (test infrastructure only). See kmeans_oracle.c for the arithmetic and its citations.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It imports nothing from the HIP package and the HIP package imports nothing from it.
"""
from .cpu import (  # noqa: F401
    assign_top2,
    bits_per_parameter,
    build,
    code_bits_per_weight,
    decode,
    inertia,
    kmeans_fit,
    parameter_counts,
    threads,
    update,
)
from . import layer  # noqa: F401,E402  (the linear layer's data path: plain numpy)
