"""Seeded workloads of the two sweeps the paper's design-space study rests on
(shapes, masks and value distributions only; nothing here packs or runs a layer).

* rate sweep: one 3x3 convolution 56x56x256 -> 256 pruned with different
  schemes at different rates (the layer of the paper's latency-vs-rate figure
  in section 4): block-punched, unstructured (1x1 blocks), whole-tensor blocks
  (the same positions punched in every filter), pattern + connectivity, and
  filter pruning (a smaller dense layer).
* block-size sweep: the 50-layer residual stack of `configs.config5` with every
  pruned layer at one rate and one block size (the axis of the paper's
  block-size study in section 4).
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

from . import configs, dtypes, masks, prng
from .configs import ACT_NONE, Layer, Workload, _tensor

RATE_SCHEMES = ("block_punched", "unstructured", "whole_tensor", "pattern", "filter")
RATES = (1, 2, 2.5, 3, 5, 7, 10)
BLOCK_SIZES = ((1, 1), (4, 4), (8, 4), (16, 8), (32, 16), (64, 64))


def rate_sweep_layer(scheme, rate, batch=1, HW=56, C=256, F=256, seed=configs.BASE_SEED + 6, dtype=dtypes.BF16):
    """The swept 3x3 layer under `scheme` at pruning rate `rate` (1 = dense)."""
    rate = Fraction(rate).limit_denominator(1000)
    xs, xe = _tensor(seed, 1, (batch, HW, HW, C), 1.0, dtype)
    Fk, lib, ids = F, None, None
    if scheme == "filter":                       # whole filters removed: a dense layer with F / rate filters
        Fk = max(4, int(round(F / float(rate) / 4.0)) * 4)
        w_store, w_exact = _tensor(seed, 100, (Fk, C, 3, 3), 0.03, dtype)
        m = masks.block_punched_mask(Fk, C, 3, 3, 8, 4, 1, seed, 1000)
        L = Layer("conv", "block_punched", C, Fk, 3, 3, 1, 1, 8, 4, float(rate), ACT_NONE, 0, -1, w_store, w_exact, m)
    elif scheme == "pattern":                    # 4 of 9 taps per kernel, whole kernels removed to reach the rate
        w_store, w_exact = _tensor(seed, 100, (F, C, 3, 3), 0.03, dtype)
        lib = masks.pattern_library(8, seed, 7)
        dead = max(0.0, 1.0 - 9.0 / (4.0 * float(rate)))
        m, ids = masks.pattern_mask(F, C, lib, dead, seed, 1000)
        L = Layer("conv", "pattern", C, F, 3, 3, 1, 1, 1, 1, float(rate), ACT_NONE, 0, -1, w_store, w_exact, m, lib, ids)
    else:
        Bf, Bc = {"block_punched": (8, 4), "unstructured": (1, 1), "whole_tensor": (F, C)}[scheme]
        w_store, w_exact = _tensor(seed, 100, (F, C, 3, 3), 0.03, dtype)
        m = masks.block_punched_mask(F, C, 3, 3, Bf, Bc, rate, seed, 1000)
        L = Layer("conv", "block_punched", C, F, 3, 3, 1, 1, Bf, Bc, float(rate), ACT_NONE, 0, -1, w_store, w_exact, m)
    L.name = "%s_r%s" % (scheme, float(rate))
    return Workload("sweep_rate_%s" % L.name, dtype, (batch, HW, HW, C), xs, xe, [L])


def inverted_residual_block(batch=64, HW=56, C=24, t=6, stride=1, Bf=8, Bc=8, rate=4, seed=configs.BASE_SEED + 7,
                            dtype=dtypes.BF16, bias=False, act=configs.ACT_RELU6):
    """The cascade "1x1 & 3x3 DW & 1x1" of the search space (section 5.1.1) in its usual
    inverted-residual form: 1x1 expansion C -> t C, ReLU6, depthwise 3x3 (stride 1 or 2), ReLU6,
    1x1 projection back to C, plus the block input when the stride is 1.  The 1x1 layers are
    block-punched at `rate`, the depthwise layer is dense.  With the defaults the outer shapes are
    those of configs.config2."""
    xs, xe = _tensor(seed, 1, (batch, HW, HW, C), 1.0, dtype)
    mid = t * C
    L1 = configs._bp_conv(seed, 0, C, mid, 1, 1, 0, Bf, Bc, rate, 0.3, dtype, act, src=0, name="expand1x1")
    dw_store, dw_exact = _tensor(seed, 150, (mid, 3, 3), 0.3, dtype)
    L2 = Layer("dwconv", "", mid, mid, 3, 3, stride, 1, 1, 1, 1.0, act, 1, -1, dw_store, dw_exact, name="dw3x3")
    L3 = configs._bp_conv(seed, 1, mid, C, 1, 1, 0, Bf, Bc, rate, 0.1, dtype, ACT_NONE, src=2,
                          res=0 if stride == 1 else -1, name="project1x1")
    if bias:  # a bias per layer (what folding a batch normalisation into the layer leaves), fp32
        for i, L in enumerate((L1, L2, L3)):
            L.bias = (0.5 * prng.normal(seed, 300 + i, L.F)).astype(np.float32)
    return Workload("inverted_residual_block", dtype, (batch, HW, HW, C), xs, xe, [L1, L2, L3])


def block_sweep_stack(Bf, Bc, rate=6, batch=1, HW=224):
    """The residual stack with every pruned conv at `rate` in Bf x Bc blocks."""
    return configs.config5(batch=batch, HW=HW, Bf=Bf, Bc=Bc, rates=(rate,))
