"""The five seeded synthetic workloads (shapes and value distributions only).

Each builder returns a `Workload`: the input tensor and a list of `Layer`
records (dense weights, mask, scheme parameters, wiring).  Nothing here runs
or packs a layer.  The workloads stand in for the paper's ImageNet-trained
networks, which are not available; the paper notes that latency does not
depend on the weight values (section 5.2.3), so random weights of the right
shape and sparsity structure measure the same thing.

Tensor numbering inside a stack: tensor 0 is the stack input, layer i writes
tensor i+1; `src` / `res` name the tensors a layer reads.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import dtypes, masks, prng

BASE_SEED = 20201200
ACT_NONE, ACT_RELU, ACT_RELU6, ACT_HARDSWISH = 0, 1, 2, 3


@dataclass
class Layer:
    kind: str                      # "conv" | "fc" | "dwconv" (depthwise 3x3, pad 1, w [C][3][3]) | "maxpool" | "avgpool"
    scheme: str = ""               # "block_punched" | "fc_block" | "pattern"
    C: int = 0
    F: int = 0
    KH: int = 1
    KW: int = 1
    stride: int = 1
    pad: int = 0
    Bf: int = 1
    Bc: int = 1
    rate: float = 1.0
    act: int = ACT_NONE
    src: int = 0
    res: int = -1
    w_store: Optional[np.ndarray] = None   # device storage (f32 or uint16 bits), [F][C][KH][KW]
    w_exact: Optional[np.ndarray] = None   # float64 values of w_store
    mask: Optional[np.ndarray] = None      # uint8, same shape
    library: Optional[np.ndarray] = None   # pattern scheme: uint8 [n_pat][9]
    pat_id: Optional[np.ndarray] = None    # pattern scheme: uint8 [F][C], 255 = removed
    name: str = ""
    bias: Optional[np.ndarray] = None      # float32 [F], added before the residual and the activation


@dataclass
class Workload:
    name: str
    dtype: int
    x_shape: tuple                 # (N, H, W, C), or (B, IN) for a lone FC layer
    x_store: np.ndarray
    x_exact: np.ndarray
    layers: List[Layer] = field(default_factory=list)

    def dense_macs(self) -> int:
        """Multiply-accumulates of the unpruned stack for the whole batch."""
        total = 0
        shapes = {0: self.x_shape}
        for i, L in enumerate(self.layers):
            s = shapes[L.src]
            if L.kind == "conv":
                N, H, W, _ = s
                Ho = (H + 2 * L.pad - L.KH) // L.stride + 1
                Wo = (W + 2 * L.pad - L.KW) // L.stride + 1
                total += N * Ho * Wo * L.F * L.C * L.KH * L.KW
                shapes[i + 1] = (N, Ho, Wo, L.F)
            elif L.kind == "fc":
                B = s[0]
                total += B * L.F * L.C
                shapes[i + 1] = (B, L.F)
            elif L.kind == "dwconv":
                N, H, W, C = s
                Ho, Wo = (H - 1) // L.stride + 1, (W - 1) // L.stride + 1
                total += N * Ho * Wo * C * 9
                shapes[i + 1] = (N, Ho, Wo, C)
            elif L.kind == "maxpool":
                N, H, W, C = s
                shapes[i + 1] = (N, (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1, C)
            elif L.kind == "avgpool":
                N, H, W, C = s
                shapes[i + 1] = (N, C)
        return total


def _tensor(seed, stream, shape, sigma, dtype):
    v = prng.normal(seed, stream, int(np.prod(shape)), sigma).reshape(shape)
    return dtypes.quantize(v, dtype)


def _bp_conv(seed, idx, C, F, k, stride, pad, Bf, Bc, rate, sigma, dtype, act, src=0, res=-1, name=""):
    w_store, w_exact = _tensor(seed, 100 + idx, (F, C, k, k), sigma, dtype)
    m = masks.block_punched_mask(F, C, k, k, Bf, Bc, rate, seed, 1000 + idx)
    return Layer("conv", "block_punched", C, F, k, k, stride, pad, Bf, Bc, float(rate), act, src, res,
                 w_store, w_exact, m, name=name)


def config1(seed=BASE_SEED + 1, H=32, W=32, C=16, F=32, Bf=4, Bc=4, rate=2, dtype=dtypes.F32):
    """One 3x3 block-punched conv, fp32, batch 1 (the small case)."""
    xs, xe = _tensor(seed, 1, (1, H, W, C), 1.0, dtype)
    L = _bp_conv(seed, 0, C, F, 3, 1, 1, Bf, Bc, rate, 0.1, dtype, ACT_NONE, name="conv3x3")
    return Workload("cfg1_conv3x3_f32", dtype, (1, H, W, C), xs, xe, [L])


def config2(seed=BASE_SEED + 2, batch=64, HW=56, C=24, mid=144, Bf=8, Bc=8, rate=4, dtype=dtypes.BF16):
    """1x1 pointwise stack C -> mid -> C with ReLU6 between (inverted-residual shape)."""
    xs, xe = _tensor(seed, 1, (batch, HW, HW, C), 1.0, dtype)
    L1 = _bp_conv(seed, 0, C, mid, 1, 1, 0, Bf, Bc, rate, 0.05, dtype, ACT_RELU6, src=0, name="expand1x1")
    L2 = _bp_conv(seed, 1, mid, C, 1, 1, 0, Bf, Bc, rate, 0.05, dtype, ACT_NONE, src=1, name="project1x1")
    return Workload("cfg2_pointwise_stack", dtype, (batch, HW, HW, C), xs, xe, [L1, L2])


def config3(seed=BASE_SEED + 3, batch=256, IN=1280, OUT=1000, Br=16, Bcol=32, rate=5, dtype=dtypes.BF16):
    """Block-based sparse FC: whole columns pruned inside Br x Bcol blocks."""
    xs, xe = _tensor(seed, 1, (batch, IN), 1.0, dtype)
    w_store, w_exact = _tensor(seed, 100, (OUT, IN, 1, 1), 0.02, dtype)
    m = masks.fc_block_mask(OUT, IN, Br, Bcol, rate, seed, 1000).reshape(OUT, IN, 1, 1)
    L = Layer("fc", "fc_block", IN, OUT, 1, 1, 1, 0, Br, Bcol, float(rate), ACT_NONE, 0, -1,
              w_store, w_exact, m, name="fc")
    return Workload("cfg3_fc_block", dtype, (batch, IN), xs, xe, [L])


def config4(seed=BASE_SEED + 4, batch=32, HW=28, C=128, F=128, n_pat=8, dead=0.3, dtype=dtypes.BF16):
    """Pattern (4 of 9 taps, centre kept) + connectivity pruned 3x3 conv."""
    xs, xe = _tensor(seed, 1, (batch, HW, HW, C), 1.0, dtype)
    w_store, w_exact = _tensor(seed, 100, (F, C, 3, 3), 0.03, dtype)
    lib = masks.pattern_library(n_pat, seed, 7)
    m, ids = masks.pattern_mask(F, C, lib, dead, seed, 1000)
    L = Layer("conv", "pattern", C, F, 3, 3, 1, 1, 1, 1, 9.0 / 4.0, ACT_NONE, 0, -1,
              w_store, w_exact, m, lib, ids, name="pattern3x3")
    return Workload("cfg4_pattern3x3", dtype, (batch, HW, HW, C), xs, xe, [L])


def config5(seed=BASE_SEED + 5, batch=1, HW=224, Bf=8, Bc=4, rates=(2, 3, 5), dtype=dtypes.BF16,
            blocks=(3, 4, 6, 3), width=64, classes=1000):
    """50-layer bottleneck residual stack (stem 7x7/2, 3x3/2 max-pool, stages of
    1x1-3x3-1x1 blocks with projection shortcuts, global average pool, FC);
    every conv block-punched with Bf x Bc blocks at a per-layer rate drawn from
    `rates`, the classifier block-based 16x32.  `width`, `HW`, `blocks` shrink it
    for tests."""
    xs, xe = _tensor(seed, 1, (batch, HW, HW, 3), 1.0, dtype)
    layers: List[Layer] = []
    draw = prng.u64(seed, 99, 256)
    n_conv = [0]

    def conv(C, F, k, stride, pad, act, src, res=-1, scale=1.0, name=""):
        i = n_conv[0]
        n_conv[0] += 1
        r = rates[int(draw[i] % np.uint64(len(rates)))]
        sigma = scale * float(np.sqrt(2.0 * r / (C * k * k)))
        layers.append(_bp_conv(seed, i, C, F, k, stride, pad, Bf, Bc, r, sigma, dtype, act, src, res, name))
        return len(layers)          # tensor id written

    t = conv(3, width, 7, 2, 3, ACT_RELU, 0, name="stem7x7")
    layers.append(Layer("maxpool", src=t, C=width, F=width, KH=3, KW=3, stride=2, pad=1, name="maxpool"))
    t = len(layers)
    cin = width
    for s, nb in enumerate(blocks):
        mid = width * (2 ** s)
        cout = mid * 4
        for b in range(nb):
            stride = 2 if (b == 0 and s > 0) else 1
            block_in = t
            a = conv(cin, mid, 1, 1, 0, ACT_RELU, block_in, name=f"s{s}b{b}_c1")
            a = conv(mid, mid, 3, stride, 1, ACT_RELU, a, name=f"s{s}b{b}_c2")
            if b == 0:
                sc = conv(cin, cout, 1, stride, 0, ACT_NONE, block_in, name=f"s{s}b{b}_sc")
            else:
                sc = block_in
            t = conv(mid, cout, 1, 1, 0, ACT_RELU, a, res=sc, scale=0.25, name=f"s{s}b{b}_c3")
            cin = cout
    layers.append(Layer("avgpool", src=t, C=cin, F=cin, name="avgpool"))
    t = len(layers)
    r = rates[int(draw[255] % np.uint64(len(rates)))]
    w_store, w_exact = _tensor(seed, 100 + 255, (classes, cin, 1, 1), float(np.sqrt(1.0 * r / cin)), dtype)
    m = masks.fc_block_mask(classes, cin, 16, 32, r, seed, 1000 + 255).reshape(classes, cin, 1, 1)
    layers.append(Layer("fc", "fc_block", cin, classes, 1, 1, 1, 0, 16, 32, float(r), ACT_NONE, t, -1,
                        w_store, w_exact, m, name="fc"))
    return Workload("cfg5_residual50", dtype, (batch, HW, HW, 3), xs, xe, layers)
