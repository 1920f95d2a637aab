"""Seeded synthetic planning inputs (layer profiles and job arguments).

This package only *generates data*.  It holds none of the planning method's
arithmetic, so both the CPU oracle and the HIP path may be fed from it.
"""
from .synthetic import (  # noqa: F401
    PlanInput,
    SplitMix64,
    config,
    config_names,
    make_profile,
    random_small,
)
from .failures import failure_draws, starting_pipelines  # noqa: F401,E402
