"""Seeded synthetic inputs for the PSA decode path (no arithmetic of the method lives here)."""
from .generator import (CONFIGS, LayerInputs, WorkloadConfig, add_headroom, as_bits, base_seed,
                        generate_layer, get_config, step_inputs)

__all__ = ["CONFIGS", "LayerInputs", "WorkloadConfig", "add_headroom", "as_bits", "base_seed",
           "generate_layer", "get_config", "step_inputs"]
