"""Seeded synthetic input generators shared by the tests, the benchmark and the CPU checker.

This package produces *inputs only* (raw feature IDs, field layouts, upstream
gradients, feature declarations).  It contains none of the arithmetic of the
embedding path itself: no tagging, no deduplication, no hashing of table slots,
no row initialisation, no optimizer maths.
"""
from .gen import (  # noqa: F401
    FeatureDecl,
    Workload,
    bounded_zipf_ranks,
    scramble_bits,
    unscramble_bits,
    make_config,
    normal_grads,
    small_int_grads,
)
from .layout import merged_inputs  # noqa: F401
