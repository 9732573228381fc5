"""CPU oracle (test infrastructure only): see sparbit_oracle.c for what it simulates.

Only tests, ``__graft_entry__.smoke()`` and the benchmark's cpu_baseline leg may
import this package.  It never imports the HIP package.
"""
from .binding import (  # noqa: F401
    ALGOS,
    BRUCK,
    NAIVE,
    RECURSIVE_DOUBLING,
    RING,
    SPARBIT,
    OracleError,
    OracleRun,
    allgather,
    allgatherv,
    build,
    naive_allgather,
    num_steps,
)
