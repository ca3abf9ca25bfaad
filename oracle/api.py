"""ctypes wrappers around oracle/npas_oracle.c plus the stack walker.

All tensors are float64 NumPy arrays holding values that are exactly
representable in the layer's storage type; the oracle accumulates in float64
and rounds a layer's output to the storage type only where a following layer
(or the caller) asks for it.  This mirrors what the masked-dense definition of
the pruned layers (paper sections 2.1 and 3) computes; nothing here is shared
with the HIP path.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "npas_oracle.c")
_LIB = os.path.join(_HERE, "libnpas_oracle.so")

ACT_NONE, ACT_RELU, ACT_RELU6, ACT_HARDSWISH = 0, 1, 2, 3
F32, BF16, F16 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("oracle_round_bf16", "oracle_round_f16", "oracle_round_f32"):
            getattr(_lib, name).restype = C.c_double
            getattr(_lib, name).argtypes = [C.c_double]
    return _lib


def _p(a, t=C.c_void_p):
    return None if a is None else a.ctypes.data_as(t)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _u8(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.uint8)


def round_to(a, dtype):
    a = _f64(a)
    out = np.empty_like(a)
    lib().oracle_round_array(_p(a), _p(out), C.c_size_t(a.size), C.c_int(dtype))
    return out


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def validate_block_punched(mask, Bf, Bc) -> int:
    m = _u8(mask)
    F, Cc, KH, KW = m.shape
    return int(lib().oracle_validate_block_punched(_p(m), F, Cc, KH, KW, Bf, Bc))


def validate_fc_block(mask, Br, Bcol) -> int:
    m = _u8(mask)
    OUT, IN = m.shape[0], m.shape[1]
    return int(lib().oracle_validate_fc_block(_p(m), OUT, IN, Br, Bcol))


def validate_pattern(mask, library):
    """Returns (rc, pat_id[F][C])."""
    m, L = _u8(mask), _u8(library)
    F, Cc = m.shape[0], m.shape[1]
    ids = np.full((F, Cc), 254, dtype=np.uint8)
    rc = int(lib().oracle_validate_pattern(_p(m), F, Cc, _p(L), L.shape[0], _p(ids)))
    return rc, ids


def pack_block_punched(W, mask, Bf):
    """Canonical compact form: (grp_ptr int32[G+1], k_pos int32[K], w_compact f64[K][Bf])."""
    W, m = _f64(W), _u8(mask)
    if W.ndim == 2:
        W, m = W.reshape(*W.shape, 1, 1), m.reshape(*m.shape, 1, 1)
    F, Cc, KH, KW = W.shape
    G = -(-F // Bf)
    total = C.c_int64(0)
    rc = lib().oracle_pack_block_punched(_p(W), _p(m), F, Cc, KH, KW, Bf, None, None, None, C.byref(total))
    assert rc == 0, rc
    K = total.value
    grp = np.zeros(G + 1, dtype=np.int32)
    kpos = np.zeros(K, dtype=np.int32)
    wc = np.zeros((K, Bf), dtype=np.float64)
    rc = lib().oracle_pack_block_punched(_p(W), _p(m), F, Cc, KH, KW, Bf, _p(grp), _p(kpos), _p(wc),
                                         C.byref(total))
    assert rc == 0, rc
    return grp, kpos, wc


def pack_pattern(W, mask):
    W, m = _f64(W), _u8(mask)
    F, Cc = W.shape[0], W.shape[1]
    w4 = np.zeros((F, Cc, 4), dtype=np.float64)
    rc = lib().oracle_pack_pattern(_p(W), _p(m), F, Cc, _p(w4))
    assert rc == 0, rc
    return w4


def conv2d_masked(X, W, mask, stride=1, pad=0, bias=None, residual=None, act=ACT_NONE):
    X, W, m, bias, residual = _f64(X), _f64(W), _u8(mask), _f64(bias), _f64(residual)
    N, H, Wd, Cc = X.shape
    F, C2, KH, KW = W.shape
    assert C2 == Cc and m.shape == W.shape
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (Wd + 2 * pad - KW) // stride + 1
    Y = np.empty((N, Ho, Wo, F), dtype=np.float64)
    if residual is not None:
        assert residual.shape == Y.shape
    rc = lib().oracle_conv2d_masked(_p(X), _p(W), _p(m), _p(bias), _p(residual), N, H, Wd, Cc, F, KH, KW,
                                    stride, pad, act, _p(Y))
    assert rc == 0, rc
    return Y


def fc_masked(X, W, mask, bias=None, act=ACT_NONE):
    X, W, m, bias = _f64(X), _f64(W), _u8(mask), _f64(bias)
    B, IN = X.shape
    OUT = W.shape[0]
    W, m = W.reshape(OUT, IN), m.reshape(OUT, IN)
    Y = np.empty((B, OUT), dtype=np.float64)
    rc = lib().oracle_fc_masked(_p(X), _p(W), _p(m), _p(bias), B, IN, OUT, act, _p(Y))
    assert rc == 0, rc
    return Y


def conv2d_pattern(X, w4, pat_id, library, stride=1, pad=1, bias=None, act=ACT_NONE):
    X, w4, ids, L, bias = _f64(X), _f64(w4), _u8(pat_id), _u8(library), _f64(bias)
    N, H, Wd, Cc = X.shape
    F = ids.shape[0]
    Ho, Wo = (H + 2 * pad - 3) // stride + 1, (Wd + 2 * pad - 3) // stride + 1
    Y = np.empty((N, Ho, Wo, F), dtype=np.float64)
    rc = lib().oracle_conv2d_pattern(_p(X), _p(w4), _p(ids), _p(L), L.shape[0], _p(bias), N, H, Wd, Cc, F,
                                     stride, pad, act, _p(Y))
    assert rc == 0, rc
    return Y


def dwconv3x3(X, W, stride=1, bias=None, residual=None, act=ACT_NONE):
    """Depthwise 3x3 convolution, padding 1; W is [C][3][3]."""
    X, W, bias, residual = _f64(X), _f64(W), _f64(bias), _f64(residual)
    N, H, Wd, Cc = X.shape
    assert W.shape == (Cc, 3, 3)
    Y = np.empty((N, (H - 1) // stride + 1, (Wd - 1) // stride + 1, Cc), dtype=np.float64)
    if residual is not None:
        assert residual.shape == Y.shape
    rc = lib().oracle_dwconv3x3(_p(X), _p(W), _p(bias), _p(residual), N, H, Wd, Cc, stride, act, _p(Y))
    assert rc == 0, rc
    return Y


def maxpool3x3s2(X):
    X = _f64(X)
    N, H, Wd, Cc = X.shape
    Y = np.empty((N, (H - 1) // 2 + 1, (Wd - 1) // 2 + 1, Cc), dtype=np.float64)
    assert lib().oracle_maxpool3x3s2(_p(X), N, H, Wd, Cc, _p(Y)) == 0
    return Y


def global_avgpool(X):
    X = _f64(X)
    N, H, Wd, Cc = X.shape
    Y = np.empty((N, Cc), dtype=np.float64)
    assert lib().oracle_global_avgpool(_p(X), N, H, Wd, Cc, _p(Y)) == 0
    return Y


def run_layer(L, tensors, dtype):
    """One layer of a stack on already-rounded inputs; returns the unrounded
    float64 output.  `L` is any object with the workload Layer fields."""
    x = tensors[L.src]
    bias = getattr(L, "bias", None)  # per output channel, part of the layer like its weights
    if L.kind == "conv":
        res = tensors[L.res] if L.res >= 0 else None
        return conv2d_masked(x, L.w_exact, L.mask, L.stride, L.pad, bias, res, L.act)
    if L.kind == "fc":
        return fc_masked(x, L.w_exact, L.mask, bias, L.act)
    if L.kind == "dwconv":
        res = tensors[L.res] if L.res >= 0 else None
        return dwconv3x3(x, L.w_exact, L.stride, bias, res, L.act)
    if L.kind == "maxpool":
        return maxpool3x3s2(x)
    if L.kind == "avgpool":
        return global_avgpool(x)
    raise ValueError(L.kind)


def run_stack(x_exact, layers, dtype):
    """Walk a layer stack.  Each layer's float64 result is rounded to the storage
    type (round-to-nearest-even) before any later layer reads it, as a device
    that stores activations in that type must.  Returns (rounded, unrounded):
    lists indexed by tensor id (tensor 0 = input)."""
    rounded = [np.asarray(x_exact, dtype=np.float64)]
    raw = [rounded[0]]
    for L in layers:
        y = run_layer(L, rounded, dtype)
        raw.append(y)
        rounded.append(round_to(y, dtype))
    return rounded, raw
