"""Seeded synthetic inputs for the MoE layer (forward inputs and upstream gradients).

This module serves the HIP library's tests, the benchmark and the CPU oracle's
tests alike.  It holds none of the layer's arithmetic and imports neither side.
"""
from .configs import CONFIGS, MoEConfig, get_config
from .generate import (MoEInputs, make_inputs, make_upstream, make_encoder_weights,
                       ExpertWeightsF64)

__all__ = ["CONFIGS", "MoEConfig", "get_config", "MoEInputs", "make_inputs", "make_upstream", "make_encoder_weights",
           "ExpertWeightsF64"]
