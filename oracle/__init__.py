"""Plain fp64 CPU oracle for the R-TOSS hot path.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the CPU-baseline leg of
the benchmark.  Nothing in the product package may import this, and this package imports
nothing from the product package.
"""
from .oracle import (  # noqa: F401
    RULE_ALL,
    RULE_ANYPAIR4,
    RULE_CONNECTED4,
    RULE_CONNECTED8,
    build,
    ACT_NONE,
    ACT_RELU,
    ACT_SILU,
    conv2d,
    conv2d_fused,
    conv2d_live3x3,
    conv2d_points,
    histogram,
    mask,
    pattern_dict,
    reduce_dict,
    select,
    threads,
)
