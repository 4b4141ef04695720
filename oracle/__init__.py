"""CPU oracle for the IntAttention pipeline -- TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may
import this package.  It shares nothing with the HIP library.
"""
from .oracle import (  # noqa: F401
    build,
    c_int,
    forward,
    forward_groups,
    forward_row_groups,
    index_map,
    index_softmax,
    lut,
    prob,
    quantize,
    quantize_row_groups,
    requant_params,
    rows,
)
