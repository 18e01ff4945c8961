"""Seeded synthetic workloads (dense, 2-D convolutional, 1-D convolutional).

This package only draws inputs (weights, biases, data). It contains none of the
gradient method's arithmetic and is the single piece of code that both the CPU
oracle's tests and the HIP path's tests and benchmark feed from.
"""
from .mlp import (CONFIGS, MLPWorkload, config_widths, haar_orthonormal_columns,
                  make_mlp, make_mlp_on_device, make_config, moonwalk_flops, backprop_flops, workload_to_host)

from .conv import (ConvWorkload, make_convnet, make_convnet_on_device, conv_out_side, conv_moonwalk_flops,
                   conv_backprop_flops, CONV_CONFIGS)

from .conv1d import FragWorkload, make_fragnet, frag_moonwalk_flops, frag_backprop_flops, FRAG_CONFIGS

__all__ = ["FragWorkload", "make_fragnet", "frag_moonwalk_flops", "frag_backprop_flops", "FRAG_CONFIGS", "ConvWorkload", "make_convnet", "make_convnet_on_device", "CONV_CONFIGS", "conv_out_side", "conv_moonwalk_flops", "conv_backprop_flops",
           "CONFIGS", "MLPWorkload", "config_widths", "haar_orthonormal_columns",
           "make_mlp", "make_mlp_on_device", "make_config", "moonwalk_flops", "backprop_flops", "workload_to_host"]
