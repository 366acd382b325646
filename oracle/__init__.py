"""fp64 CPU oracle for the KurTail rotation-learning step (test infrastructure).

This package is NOT part of the product.  Only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may import it.  It wraps ``kt_oracle.c``
(plain C, double precision, OpenMP over token rows) through ctypes and shares no
code with the HIP path.  See the header of ``kt_oracle.c`` for the passage of
the paper each function follows and for how it is pinned.
"""
from .binding import (  # noqa: F401
    build_oracle,
    num_threads,
    rotate,
    row_moments,
    loss_grad,
    pooled_loss_grad,
    cayley_step,
    cayley_step_right,
    cayley_adam_step,
    fakequant_int4,
    quant_metrics,
    quant_sensitivity,
    quant_mse,
    hadamard_rows,
    hadamard_factor,
    hadamard_matrix,
    fuse_rotation,
)
