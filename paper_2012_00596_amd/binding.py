from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_LIB = os.path.join(_HERE, "libnpas.so")
SOURCES = ["pack.cpp", "api.cpp", "kernels.hip", "spatial_kernels.hip", "small_kernels.hip", "block_kernels.hip", "noalloc.hip"]
HEADER = os.path.join(os.path.dirname(_HERE), "include", "npas.h")

F32, BF16, F16 = 0, 1, 2
ACT_NONE, ACT_RELU, ACT_RELU6, ACT_HARDSWISH = 0, 1, 2, 3
SCHEME_BLOCK_PUNCHED, SCHEME_FC_BLOCK, SCHEME_PATTERN, SCHEME_DEPTHWISE = 0, 1, 2, 3
LAYER_CONV, LAYER_FC, LAYER_MAXPOOL3X3S2, LAYER_GLOBAL_AVGPOOL, LAYER_DEPTHWISE3X3 = 0, 1, 2, 3, 4
STACK_FUSE_POINTWISE = 1
STACK_FUSE_INVERTED_RESIDUAL = 2
STACK_FUSE_CONV_MAXPOOL = 4
OK, E_NULL, E_SHAPE, E_MASK_NOT_BLOCK_UNIFORM, E_MASK_NOT_IN_LIBRARY, E_DTYPE, E_WORKSPACE, E_HIP, E_MASK_VALUE = \
    0, -1, -2, -3, -4, -5, -6, -7, -8

EXPORTS = [
    "npas_last_error", "npas_pack_block_punched", "npas_pack_fc_block", "npas_pack_pattern",
    "npas_pack_depthwise3x3", "npas_depthwise3x3",
    "npas_packed_info", "npas_packed_export", "npas_free", "npas_conv2d_sparse", "npas_conv2d_kernel_name",
    "npas_fc_sparse",
    "npas_maxpool3x3s2", "npas_global_avgpool", "npas_stack_create", "npas_stack_workspace_bytes",
    "npas_run_stack", "npas_stack_num_launches", "npas_stack_free", "npas_stack_describe", "npas_debug_set_switches",
    "npas_run_stack_static", "npas_debug_launch_empty",
]
STATIC_WORKSPACE_BYTES = 32 << 20
DESCRIBE_COLS = 11


class NpasError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libnpas error {code}: {msg}")
        self.code = code


def build(force: bool = True) -> str:
    """Compile libnpas.so for gfx950 in-tree with hipcc (one object per source, compiled side by side)."""
    from concurrent.futures import ThreadPoolExecutor
    srcs = [os.path.join(_CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(_CSRC, "npas_internal.h"), os.path.join(_CSRC, "device_util.h"), HEADER]
    if not force and os.path.exists(_LIB) and all(os.path.getmtime(_LIB) >= os.path.getmtime(d) for d in deps):
        return _LIB
    flags = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, os.path.basename(s) + ".o") for s in srcs]

    def compile_one(pair):
        src, obj = pair
        if force or not os.path.exists(obj) or any(os.path.getmtime(obj) < os.path.getmtime(d) for d in [src] + deps[len(srcs):]):
            subprocess.check_call(["hipcc"] + flags + ["-c", src, "-o", obj])

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        list(pool.map(compile_one, zip(srcs, objs)))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", _LIB] + objs)
    return _LIB


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("packed", C.c_void_p), ("stride", C.c_int), ("pad", C.c_int),
                ("act", C.c_int), ("src", C.c_int), ("res", C.c_int), ("bias_dev", C.c_void_p)]


_lib = None


def lib():
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise RuntimeError(f"{_LIB} is missing: run __graft_entry__.build() (hipcc, gfx950) first; "
                               "there is no fallback path")
        L = C.CDLL(_LIB)
        L.npas_last_error.restype = C.c_char_p
        vp, ip = C.c_void_p, C.c_int
        L.npas_pack_block_punched.argtypes = [vp, vp, ip, ip, ip, ip, ip, ip, ip, vp, C.POINTER(vp)]
        L.npas_pack_fc_block.argtypes = [vp, vp, ip, ip, ip, ip, ip, vp, C.POINTER(vp)]
        L.npas_pack_pattern.argtypes = [vp, vp, ip, ip, vp, ip, ip, vp, C.POINTER(vp)]
        L.npas_pack_depthwise3x3.argtypes = [vp, ip, ip, vp, C.POINTER(vp)]
        L.npas_depthwise3x3.argtypes = [vp, vp, vp, ip, ip, ip, ip, vp, vp, ip, vp]
        L.npas_packed_info.argtypes = [vp, vp]
        L.npas_packed_export.argtypes = [vp, vp, vp, vp, vp, vp]
        L.npas_free.argtypes = [vp]
        L.npas_free.restype = None
        L.npas_conv2d_sparse.argtypes = [vp, vp, vp, ip, ip, ip, ip, ip, vp, vp, ip, vp]
        L.npas_conv2d_kernel_name.argtypes = [vp, ip, ip, ip, ip, ip]
        L.npas_conv2d_kernel_name.restype = C.c_char_p
        L.npas_fc_sparse.argtypes = [vp, vp, vp, ip, vp, ip, vp]
        L.npas_maxpool3x3s2.argtypes = [vp, vp, ip, ip, ip, ip, ip, vp]
        L.npas_global_avgpool.argtypes = [vp, vp, ip, ip, ip, ip, ip, vp]
        L.npas_stack_create.argtypes = [C.POINTER(LayerDesc), ip, ip, ip, C.c_uint, C.POINTER(vp)]
        L.npas_stack_workspace_bytes.argtypes = [vp, ip]
        L.npas_stack_workspace_bytes.restype = C.c_size_t
        L.npas_run_stack.argtypes = [vp, vp, vp, ip, vp, C.c_size_t, vp]
        L.npas_stack_num_launches.argtypes = [vp]
        L.npas_stack_free.argtypes = [vp]
        L.npas_stack_free.restype = None
        L.npas_stack_describe.argtypes = [vp, ip, vp, ip]
        L.npas_run_stack_static.argtypes = [vp, vp, vp, ip, vp]
        L.npas_debug_launch_empty.argtypes = [ip, vp]
        L.npas_debug_set_switches.argtypes = [C.c_char_p, ip]
        L.npas_debug_set_switches.restype = None
        _lib = L
    return _lib


def last_error() -> str:
    return lib().npas_last_error().decode()


def set_switches(force_variant=None, no_balance=False):
    """Testing aid: replaces NPAS_FORCE_VARIANT / NPAS_NO_BALANCE for this process (None = no override)."""
    lib().npas_debug_set_switches(force_variant.encode() if force_variant else None, 1 if no_balance else 0)


def launch_empty(count, stream=None):
    """Measurement aid: `count` launches of an empty kernel on the stream."""
    _check(lib().npas_debug_launch_empty(count, stream))


def _check(rc):
    if rc != 0:
        raise NpasError(rc, last_error())


def _host(a):
    """Host pointer of a contiguous NumPy array (or None)."""
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def _dev(t):
    """Device pointer: a torch tensor, an int address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous()
    return t.data_ptr()


def _np_storage(dtype):
    return np.float32 if dtype == F32 else np.uint16


class Packed:
    """Owner of one npas_packed handle."""

    def __init__(self, handle):
        self.handle = handle

    def __del__(self):
        if getattr(self, "handle", None):
            lib().npas_free(self.handle)
            self.handle = None

    def info(self):
        v = np.zeros(16, dtype=np.int64)
        _check(lib().npas_packed_info(self.handle, _host(v)))
        keys = ["scheme", "dtype", "F", "C", "KH", "KW", "Bf", "Bc", "G", "K_total", "n_pat", "device_ready",
                "variant", "device_bytes", "compact_weight_bytes", "reserved"]
        return dict(zip(keys, (int(x) for x in v)))

    def export(self):
        """Canonical compact form as NumPy arrays (storage-type bit patterns for weights)."""
        i = self.info()
        grp = np.zeros(i["G"] + 1, dtype=np.int32)
        kpos = np.zeros(i["K_total"], dtype=np.int32)
        wc = np.zeros((i["C"], 9) if i["scheme"] == SCHEME_DEPTHWISE else (i["K_total"], i["Bf"]),
                      dtype=_np_storage(i["dtype"]))
        out = {"grp_ptr": grp, "k_pos": kpos, "w_compact": wc}
        pat = w4 = None
        if i["scheme"] == SCHEME_PATTERN:
            pat = np.zeros((i["F"], i["C"]), dtype=np.uint8)
            w4 = np.zeros((i["F"], i["C"], 4), dtype=_np_storage(i["dtype"]))
            out.update(pat_id=pat, w4=w4)
        _check(lib().npas_packed_export(self.handle, _host(grp), _host(kpos), _host(wc), _host(pat), _host(w4)))
        return out


def pack_block_punched(w, mask, Bf, Bc, dtype, stream=None):
    """w: NumPy [F][C][KH][KW] in storage type (float32, or uint16 bits); mask uint8 same shape."""
    F, Cc, KH, KW = w.shape
    h = C.c_void_p()
    _check(lib().npas_pack_block_punched(_host(w), _host(mask), F, Cc, KH, KW, Bf, Bc, dtype, stream, C.byref(h)))
    return Packed(h)


def pack_fc_block(w, mask, Br, Bcol, dtype, stream=None):
    OUT, IN = w.shape[0], w.shape[1]
    h = C.c_void_p()
    _check(lib().npas_pack_fc_block(_host(w), _host(mask), OUT, IN, Br, Bcol, dtype, stream, C.byref(h)))
    return Packed(h)


def pack_pattern(w, mask, library, dtype, stream=None):
    F, Cc = w.shape[0], w.shape[1]
    h = C.c_void_p()
    _check(lib().npas_pack_pattern(_host(w), _host(mask), F, Cc, _host(library), library.shape[0], dtype, stream,
                                   C.byref(h)))
    return Packed(h)


def pack_depthwise3x3(w, dtype, stream=None):
    """w: [C][3][3] in the storage type (float32, or uint16 bit patterns)."""
    w = np.ascontiguousarray(w, dtype=_np_storage(dtype))
    assert w.ndim == 3 and w.shape[1:] == (3, 3)
    h = C.c_void_p()
    _check(lib().npas_pack_depthwise3x3(_host(w), w.shape[0], dtype, stream, C.byref(h)))
    return Packed(h)


def depthwise3x3(packed, x, y, N, H, W, stride, bias=None, residual=None, act=ACT_NONE, stream=None):
    _check(lib().npas_depthwise3x3(packed.handle, _dev(x), _dev(y), N, H, W, stride, _dev(bias), _dev(residual), act,
                                   stream))


def conv2d_sparse(packed, x, y, N, H, W, stride, pad, bias=None, residual=None, act=ACT_NONE, stream=None):
    _check(lib().npas_conv2d_sparse(packed.handle, _dev(x), _dev(y), N, H, W, stride, pad, _dev(bias),
                                    _dev(residual), act, stream))


def conv2d_kernel_name(packed, N, H, W, stride, pad):
    name = lib().npas_conv2d_kernel_name(packed.handle, N, H, W, stride, pad)
    return name.decode() if name else None


def fc_sparse(packed, x, y, B, bias=None, act=ACT_NONE, stream=None):
    _check(lib().npas_fc_sparse(packed.handle, _dev(x), _dev(y), B, _dev(bias), act, stream))


def maxpool3x3s2(x, y, N, H, W, Cc, dtype, stream=None):
    _check(lib().npas_maxpool3x3s2(_dev(x), _dev(y), N, H, W, Cc, dtype, stream))


def global_avgpool(x, y, N, H, W, Cc, dtype, stream=None):
    _check(lib().npas_global_avgpool(_dev(x), _dev(y), N, H, W, Cc, dtype, stream))


class Stack:
    """Owner of one npas_stack handle (keeps its packed layers alive)."""

    def __init__(self, layers, H, W, flags=0):
        """layers: list of dicts {kind, packed (Packed|None), stride, pad, act, src, res, bias}."""
        n = len(layers)
        arr = (LayerDesc * n)()
        self._keep = []
        for i, L in enumerate(layers):
            p = L.get("packed")
            self._keep.append(p)
            arr[i] = LayerDesc(L["kind"], p.handle if p is not None else None, L.get("stride", 1), L.get("pad", 0),
                               L.get("act", ACT_NONE), L.get("src", i), L.get("res", -1), _dev(L.get("bias")))
        h = C.c_void_p()
        _check(lib().npas_stack_create(arr, n, H, W, flags, C.byref(h)))
        self.handle = h

    def __del__(self):
        if getattr(self, "handle", None):
            lib().npas_stack_free(self.handle)
            self.handle = None

    def workspace_bytes(self, N):
        return int(lib().npas_stack_workspace_bytes(self.handle, N))

    def num_launches(self):
        return int(lib().npas_stack_num_launches(self.handle))

    def run_static(self, x, y, N, stream=None):
        """npas_run_stack_static: the library's own static workspace, no allocation."""
        _check(lib().npas_run_stack_static(self.handle, _dev(x), _dev(y), N, stream))

    def describe(self, N):
        """The launches of one run at batch N: list of dicts (see npas_stack_describe in include/npas.h)."""
        n = self.num_launches()
        rows = np.zeros((max(n, 1), DESCRIBE_COLS), dtype=np.int64)
        got = lib().npas_stack_describe(self.handle, N, _host(rows), n)
        if got < 0:
            _check(got)
        keys = ["first", "last", "src", "res", "out", "off_src", "off_res", "off_out", "bytes_src", "bytes_res", "bytes_out"]
        return [dict(zip(keys, (int(v) for v in rows[i]))) for i in range(got)]

    def run(self, x, y, N, workspace, workspace_bytes, stream=None):
        _check(lib().npas_run_stack(self.handle, _dev(x), _dev(y), N, _dev(workspace), workspace_bytes, stream))
