"""fp64 CPU oracle of the K-FAC preconditioner step (test infrastructure only).

The arithmetic lives in ``kfac_oracle.c``; this module only marshals numpy
arrays into it.  Nothing in the product package may import this module: it
exists for the tests, the smoke check and the benchmark's CPU-baseline leg.
"""
from .kfac_oracle import (  # noqa: F401
    build,
    num_threads,
    kron,
    unfold,
    gram,
    gram_entry,
    conv_factor_entry,
    ema,
    eigh,
    eigh_jacobi,
    eigh_tridiag,
    precondition,
    bruteforce,
    spd_solve,
    schedule,
    grad_scale,
    precondition_inverse,
)
