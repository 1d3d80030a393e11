"""CPU checker for the densify path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the GPU library and its Python binding never do.
"""
from . import accumulate  # noqa: F401
from .reference import (  # noqa: F401
    OracleResult,
    buffer_bytes,
    densify,
    densify_one_shot,
    densify_timed,
    unique_ids,
)
