"""Layer lists of the benchmark configurations (shapes only) and model instantiation.

A model is a list of `Layer` records.  Each hidden layer is
conv/FC -> step (threshold + sign) -> optional 2x2 max-pool; the last FC emits int32
logits and has no step.  Shapes follow the model tables of the paper (Tab. I, Tab. II)
as re-stated by the benchmark configurations: a 28x28x1 small CNN and a 32x32x3
VGG-small, plus an all-FC MLP.
"""
from dataclasses import dataclass, field
from typing import List, Optional
import numpy as np

from . import gen

KIND_CONV_FIRST = "conv_first_int8"   # int8 activations x +-1 weights
KIND_CONV_BIN = "conv_binary"         # +-1 x +-1, 3x3, stride 1, pad 1 (pad = -1)
KIND_FC_BIN = "fc_binary"             # +-1 x +-1 dense


@dataclass
class Layer:
    kind: str
    c_in: int
    c_out: int
    kh: int = 1
    kw: int = 1
    pad: int = 0
    step: bool = True       # threshold + sign after the layer
    pool: int = 1           # 1 = none, 2 = 2x2 stride-2 max-pool after the step
    # filled by build_model():
    h_in: int = 0
    w_in: int = 0
    h_out: int = 0          # after pooling
    w_out: int = 0
    fan_in: int = 0
    weights: Optional[np.ndarray] = None   # int8 +-1, [c_out][kh][kw][c_in] or [c_out][k]
    thr: Optional[np.ndarray] = None       # int32 [c_out]
    flip: Optional[np.ndarray] = None      # uint8 [c_out]


def mlp_config0() -> List[Layer]:
    # FC1 consumes the flattened int8 image: a 1x1 "convolution" over 784 channels.
    return [
        Layer(KIND_CONV_FIRST, 784, 512, 1, 1, 0),
        Layer(KIND_FC_BIN, 512, 512),
        Layer(KIND_FC_BIN, 512, 10, step=False),
    ]


def small_cnn_config1() -> List[Layer]:
    return [
        Layer(KIND_CONV_FIRST, 1, 64, 3, 3, 1, pool=2),
        Layer(KIND_CONV_BIN, 64, 64, 3, 3, 1, pool=2),
        Layer(KIND_FC_BIN, 3136, 2048),
        Layer(KIND_FC_BIN, 2048, 10, step=False),
    ]


def vgg_small_config2() -> List[Layer]:
    return [
        Layer(KIND_CONV_FIRST, 3, 128, 3, 3, 1),
        Layer(KIND_CONV_BIN, 128, 128, 3, 3, 1, pool=2),
        Layer(KIND_CONV_BIN, 128, 256, 3, 3, 1),
        Layer(KIND_CONV_BIN, 256, 256, 3, 3, 1, pool=2),
        Layer(KIND_CONV_BIN, 256, 512, 3, 3, 1),
        Layer(KIND_CONV_BIN, 512, 512, 3, 3, 1, pool=2),
        Layer(KIND_FC_BIN, 8192, 1024),
        Layer(KIND_FC_BIN, 1024, 1024),
        Layer(KIND_FC_BIN, 1024, 10, step=False),
    ]


_MODELS = {
    "mlp": (0, mlp_config0, (1, 1, 784)),
    "small_cnn": (1, small_cnn_config1, (28, 28, 1)),
    "vgg_small": (2, vgg_small_config2, (32, 32, 3)),
}

# (M, N, K) of the isolated binary GEMM sweep.
GEMM_SWEEP_SHAPES = [(1024, 1024, 1024), (4096, 4096, 4096), (8192, 8192, 8192),
                     (16384, 16384, 16384), (1, 8192, 8192)]

# (H=W, C_in=C_out) of the per-layer conv3x3 sweep at batch 1024.
CONV_SWEEP_SHAPES = [(hw, c) for hw in (8, 16, 32) for c in (128, 256, 512)]


def build_model(layers: List[Layer], in_h: int, in_w: int, in_c: int, config_id: int) -> List[Layer]:
    """Fill in spatial shapes and draw weights / thresholds / flips for every layer."""
    h, w, c = in_h, in_w, in_c
    flat = False
    for li, L in enumerate(layers):
        if L.kind == KIND_FC_BIN:
            if not flat:
                k = h * w * c
                h, w, c = 1, 1, k
                flat = True
            assert L.c_in == c, (li, L.c_in, c)
            L.h_in, L.w_in = 1, 1
            L.fan_in = L.c_in
            wshape = (L.c_out, L.c_in)
        else:
            assert L.c_in == c, (li, L.c_in, c)
            L.h_in, L.w_in = h, w
            L.fan_in = L.kh * L.kw * L.c_in
            wshape = (L.c_out, L.kh, L.kw, L.c_in)
        ho = L.h_in + 2 * L.pad - L.kh + 1
        wo = L.w_in + 2 * L.pad - L.kw + 1
        L.h_out, L.w_out = ho // L.pool, wo // L.pool
        L.weights = gen.draw_pm1(gen.rng_for(config_id, li, gen.T_WEIGHT), wshape)
        if L.step:
            L.thr = gen.draw_threshold(gen.rng_for(config_id, li, gen.T_THR), L.c_out, L.fan_in)
            L.flip = gen.draw_flip(gen.rng_for(config_id, li, gen.T_FLIP), L.c_out)
        h, w, c = L.h_out, L.w_out, L.c_out
    return layers


def model_by_name(name: str):
    """Returns (config_id, layers with tensors drawn, (in_h, in_w, in_c))."""
    cid, fn, (ih, iw, ic) = _MODELS[name]
    layers = build_model(fn(), ih, iw, ic, cid)
    return cid, layers, (ih, iw, ic)


def model_binary_macs(layers: List[Layer]) -> int:
    """+-1 x +-1 multiply-accumulates per image."""
    t = 0
    for L in layers:
        if L.kind != KIND_CONV_FIRST:
            t += L.h_out * L.pool * L.w_out * L.pool * L.c_out * L.fan_in
    return t


def model_int8_macs(layers: List[Layer]) -> int:
    t = 0
    for L in layers:
        if L.kind == KIND_CONV_FIRST:
            t += L.h_out * L.pool * L.w_out * L.pool * L.c_out * L.fan_in
    return t
