"""fp64 CPU oracle for the GKA layer forward pass (test infrastructure, not product code).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It shares nothing with the HIP library.
"""
from .gka_oracle import (  # noqa: F401
    build,
    forward,
    decode_step,
    chebyshev,
    omega_schedule,
    cholesky_solve,
    num_threads,
    SOLVER_CHEBYSHEV,
    SOLVER_CHOLESKY,
)
