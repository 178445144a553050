"""Seeded synthetic inputs shared by the oracle tests and the HIP path.

This package produces *inputs only* (datasets, labels, initial parameters,
flat stress vectors, quadratic problem constants).  It contains none of the
method's arithmetic: no SGD step, no averaging, no controller, no index
stream.  Both sides of every parity test take their inputs from here so that
they start from identical bytes.
"""
from .generate import (  # noqa: F401
    CONFIGS,
    Workload,
    bf16_representable,
    flat_stress,
    gaussian_mixture,
    image_like,
    init_params,
    make_workload,
    param_count,
    quad_problem,
)
