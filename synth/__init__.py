"""Seeded synthetic workload generators.

This package describes the SuperNet families (layer names and maximum shapes),
draws their random-init weights, SubnetNorm statistics, subnet control tuples
and request inputs.  It serves both the CPU oracle's tests and the HIP path's
tests; it contains no forward-pass arithmetic and imports neither of them.
"""
from .rng import keyed_rng
from .arch import (TinySpec, ResNetSpec, MBV3Spec, TransformerSpec, SubnetCfg,
                   round_channels, MAX_STAGES, MAX_DEPTH)
from .weights import make_weights, make_stats, make_inputs, to_bf16_values
from .cfgs import enumerate_cfgs, zipf_assignment, subnet_macs

__all__ = [
    "keyed_rng", "TinySpec", "ResNetSpec", "MBV3Spec", "TransformerSpec",
    "SubnetCfg", "round_channels", "MAX_STAGES", "MAX_DEPTH", "make_weights",
    "make_stats", "make_inputs", "to_bf16_values", "enumerate_cfgs",
    "zipf_assignment", "subnet_macs",
]
