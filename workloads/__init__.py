"""Seeded synthetic MLP workloads.

This package only draws inputs (weights, biases, data). It contains none of the
gradient method's arithmetic and is the single piece of code that both the CPU
oracle's tests and the HIP path's tests and benchmark feed from.
"""
from .mlp import (CONFIGS, MLPWorkload, config_widths, haar_orthonormal_columns,
                  make_mlp, make_mlp_on_device, make_config, moonwalk_flops, backprop_flops)

__all__ = ["CONFIGS", "MLPWorkload", "config_widths", "haar_orthonormal_columns",
           "make_mlp", "make_mlp_on_device", "make_config", "moonwalk_flops", "backprop_flops"]
