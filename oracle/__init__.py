"""CPU oracle for ExDyna's gradient-selection path -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares no code with the HIP library and never imports it.
"""
from .oracle import (  # noqa: F401
    Oracle,
    allocate,
    block_size,
    build,
    estimate,
    lib_path,
    owner,
    partition,
    scale_factor,
    select,
)
