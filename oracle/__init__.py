"""Float64 CPU oracle for Soft-DTW.  Test infrastructure: the product package never imports this."""
from .sdtw_oracle import (  # noqa: F401
    build,
    batch,
    pair_tables,
    from_cost,
    barycenter_step,
    max_threads,
    normalized,
    ragged_batch,
)
