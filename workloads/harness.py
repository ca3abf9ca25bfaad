"""Plumbing between the workload records and the C-ABI binding, shared by the benchmark, the smoke
check and the GPU tests: device buffers through PyTorch, packing a `Layer`, describing a stack, running
one layer.  The binding module and torch are passed in; nothing here computes or checks anything."""
import numpy as np

from . import dtypes


def to_dev(storage, torch):
    a = np.ascontiguousarray(storage)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def new_dev(shape, dtype, torch, fill=None):
    td = torch.float32 if dtype == dtypes.F32 else torch.int16
    t = torch.empty(shape, dtype=td, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def from_dev(t, dtype):
    a = t.cpu().numpy()
    if dtype != dtypes.F32:
        a = a.view(np.uint16)
    return dtypes.storage_to_f64(a, dtype)


def pack_layer(npas, L, dtype):
    if L.kind == "dwconv":
        return npas.pack_depthwise3x3(L.w_store, dtype)
    if L.scheme == "block_punched":
        return npas.pack_block_punched(L.w_store, L.mask, L.Bf, L.Bc, dtype)
    if L.scheme == "fc_block":
        OUT, IN = L.F, L.C
        return npas.pack_fc_block(L.w_store.reshape(OUT, IN), L.mask.reshape(OUT, IN), L.Bf, L.Bc, dtype)
    if L.scheme == "pattern":
        return npas.pack_pattern(L.w_store, L.mask, L.library, dtype)
    raise ValueError(L.scheme)


def out_shape(L, in_shape):
    if L.kind == "conv":
        N, H, W, _ = in_shape
        return (N, (H + 2 * L.pad - L.KH) // L.stride + 1, (W + 2 * L.pad - L.KW) // L.stride + 1, L.F)
    if L.kind == "fc":
        return (in_shape[0], L.F)
    if L.kind == "dwconv":
        N, H, W, C = in_shape
        return (N, (H - 1) // L.stride + 1, (W - 1) // L.stride + 1, C)
    if L.kind == "maxpool":
        N, H, W, C = in_shape
        return (N, (H - 1) // 2 + 1, (W - 1) // 2 + 1, C)
    if L.kind == "avgpool":
        return (in_shape[0], in_shape[3])
    raise ValueError(L.kind)


def run_layer_gpu(npas, torch, L, packed, x_dev, in_shape, dtype, res_dev=None, bias_dev=None):
    """One layer through the C ABI; returns the device output tensor."""
    oshape = out_shape(L, in_shape)
    # poison the output so that unwritten elements show up
    y = new_dev(oshape, dtype, torch, fill=(float("nan") if dtype == dtypes.F32 else 0x7FC1))
    if L.kind == "conv":
        N, H, W, _ = in_shape
        npas.conv2d_sparse(packed, x_dev, y, N, H, W, L.stride, L.pad, bias_dev, res_dev, L.act)
    elif L.kind == "fc":
        npas.fc_sparse(packed, x_dev, y, in_shape[0], bias_dev, L.act)
    elif L.kind == "dwconv":
        N, H, W, _ = in_shape
        npas.depthwise3x3(packed, x_dev, y, N, H, W, L.stride, bias_dev, res_dev, L.act)
    elif L.kind == "maxpool":
        N, H, W, C = in_shape
        npas.maxpool3x3s2(x_dev, y, N, H, W, C, dtype)
    elif L.kind == "avgpool":
        N, H, W, C = in_shape
        npas.global_avgpool(x_dev, y, N, H, W, C, dtype)
    torch.cuda.synchronize()
    return y


def stack_descs(npas, layers, packed, biases=None):
    """Layer descriptions for npas.Stack; biases: per layer a device tensor (fp32, kept alive by the caller) or None."""
    kinds = {"conv": npas.LAYER_CONV, "fc": npas.LAYER_FC, "maxpool": npas.LAYER_MAXPOOL3X3S2,
             "avgpool": npas.LAYER_GLOBAL_AVGPOOL, "dwconv": npas.LAYER_DEPTHWISE3X3}
    return [dict(kind=kinds[L.kind], packed=packed[i], stride=L.stride, pad=L.pad, act=L.act, src=L.src, res=L.res,
                 bias=None if biases is None else biases[i])
            for i, L in enumerate(layers)]


def bias_tensors(layers, torch):
    """Per layer its bias on the device (fp32) or None."""
    return [None if getattr(L, "bias", None) is None else torch.from_numpy(np.ascontiguousarray(L.bias, dtype=np.float32)).cuda()
            for L in layers]
