"""CPU oracle for the K-FAC hot path (TEST INFRASTRUCTURE, not a product path).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP implementation and never calls it.
"""
from .kfac_oracle import (  # noqa: F401
    im2col_rows, gout_rows, factor_from_rows, running_average,
    update_factor_A, update_factor_G, damped_inverse, precondition, kfac_step,
    packed_size, pack_upper, unpack_upper, NotPositiveDefinite,
)
