"""fp64 CPU oracle (test infrastructure, not the product).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The HIP library never does.
"""
from .oracle import (  # noqa: F401
    build,
    centered_clip,
    coordinate_median,
    geometric_median,
    num_threads,
    set_num_threads,
    philox4x32_10,
    preclip_scales,
    split,
    tau_schedule,
    verification3,
    verification12,
    partition_hashes,
    verify,
    z_hat,
    z_norm,
    z_uniforms,
)
