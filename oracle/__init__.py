"""CPU oracle for the replayed kernel chain -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It is independent of the HIP path: no shared code, headers or constants.
"""
from .binding import (  # noqa: F401
    build,
    lib,
    run_chain,
    run_op,
    select,
    bf16_from_f64,
    bf16_to_f64,
    gelu_f64,
    set_threads,
    max_threads,
)
