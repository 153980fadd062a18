"""Seeded synthetic inputs for the NEZHA draft+verify path.

This package only draws numbers and lays out catalogs.  It holds none of the
method's arithmetic (no projection, softmax, beam search, key packing or
membership test); both the CPU oracle's tests and the HIP path's tests and
bench draw their inputs from here so that the two sides see identical bits.
"""
from .rng import uniform01, normal, randint, mix64, Bijection
from .configs import CONFIGS, StepConfig, get_config
from .inputs import draft_inputs, round_to_bf16
from .catalog import (uniform_catalog, zipf_catalog, planted_catalog, plant_mask,
                      absent_tuples, stress_queries, digits_of, zipf_weights)

__all__ = [
    "uniform01", "normal", "randint", "mix64", "Bijection",
    "CONFIGS", "StepConfig", "get_config",
    "draft_inputs", "round_to_bf16",
    "uniform_catalog", "zipf_catalog", "planted_catalog", "absent_tuples",
    "stress_queries", "digits_of", "zipf_weights", "plant_mask",
]
