"""Seeded synthetic inputs and layer lists for the five benchmark configurations.

This module is shared by the CPU oracle's tests and by the GPU tests / bench.  It holds
no arithmetic of the method (no dot products, thresholds applied, pooling or packing):
it only draws random tensors and lists layer shapes.
"""
from .gen import (BASE_SEED, tensor_seed, rng_for, draw_images, draw_pm1, draw_threshold,
                  draw_flip, draw_bits_pm1)
from .configs import (Layer, mlp_config0, small_cnn_config1, vgg_small_config2,
                      GEMM_SWEEP_SHAPES, CONV_SWEEP_SHAPES, build_model, model_by_name,
                      model_binary_macs, model_int8_macs)
