"""CPU-side tests of the HIP library: it loads, exports what include/npas.h
declares, packs (host logic) bit-identically to the oracle's packer, rejects
illegal masks, and fails loudly instead of computing without a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2012_00596_amd as npas
from tests import helpers
from workloads import configs, dtypes, masks, prng

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "npas.h")).read()
    declared = set(re.findall(r"\b(npas_[a-z0-9_]+)\s*\(", header))
    declared -= {"npas_packed", "npas_stack"}
    assert declared == set(npas.binding.EXPORTS)
    L = npas.lib()
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("builder,kw", [
    (configs.config1, {}),
    (configs.config2, dict(batch=1, HW=4)),
    (configs.config3, dict(batch=2)),
    (configs.config4, dict(batch=1, HW=4)),
    (configs.config5, dict(batch=1, HW=32, width=16, blocks=(1, 1, 1, 1))),
])
def test_packing_metadata_bit_exact_vs_oracle(builder, kw):
    w = builder(**kw)
    for L in w.layers:
        if L.kind not in ("conv", "fc"):
            continue
        p = helpers.pack_layer(npas, L, w.dtype)
        helpers.check_metadata(oracle, L, p, w.dtype)
        info = p.info()
        assert info["F"] == L.F and info["C"] == L.C and info["dtype"] == w.dtype


@pytest.mark.parametrize("dtype", [dtypes.F32, dtypes.BF16, dtypes.F16])
@pytest.mark.parametrize("F,C,k,Bf,Bc,rate", [(10, 7, 3, 4, 4, 2), (5, 3, 7, 8, 4, 5), (16, 16, 1, 1, 1, 3),
                                               (12, 8, 3, 12, 8, 2), (9, 40, 1, 16, 32, 5)])
def test_packing_edge_blocks_and_degenerate_sizes(dtype, F, C, k, Bf, Bc, rate):
    m = masks.block_punched_mask(F, C, k, k, Bf, Bc, rate, 31)
    store, exact = dtypes.quantize(prng.normal(5, 3, F * C * k * k).reshape(F, C, k, k), dtype)
    p = npas.pack_block_punched(store, m, Bf, Bc, dtype)
    L = configs.Layer("conv", "block_punched", C, F, k, k, 1, 0, Bf, Bc, rate, w_store=store, w_exact=exact, mask=m)
    helpers.check_metadata(oracle, L, p, dtype)
    # garbage under the mask must not leak into the compact form
    junk = store.copy()
    junk[m == 0] = 0x7FC0 if dtype != dtypes.F32 else np.nan
    e1, e2 = p.export(), npas.pack_block_punched(junk, m, Bf, Bc, dtype).export()
    for key in e1:
        np.testing.assert_array_equal(e1[key].view(np.uint8), e2[key].view(np.uint8))


def test_fc_rows_and_columns():
    OUT, IN = 40, 70
    m = masks.fc_block_mask(OUT, IN, 16, 32, 4, 9)
    m[3, :32] = 0            # a pruned row inside a block
    store, exact = dtypes.quantize(prng.normal(6, 3, OUT * IN).reshape(OUT, IN), dtypes.BF16)
    p = npas.pack_fc_block(store, m, 16, 32, dtypes.BF16)
    L = configs.Layer("fc", "fc_block", IN, OUT, 1, 1, 1, 0, 16, 32, 4, w_store=store.reshape(OUT, IN, 1, 1),
                      w_exact=exact.reshape(OUT, IN, 1, 1), mask=m.reshape(OUT, IN, 1, 1))
    helpers.check_metadata(oracle, L, p, dtypes.BF16)


def test_illegal_masks_are_rejected_not_repaired():
    F, C = 8, 8
    w = np.zeros((F, C, 3, 3), dtype=np.float32)
    m = masks.block_punched_mask(F, C, 3, 3, 4, 4, 2, 16)
    bad = m.copy()
    bad[1, 2, 1, 1] ^= 1
    with pytest.raises(npas.NpasError) as e:
        npas.pack_block_punched(w, bad, 4, 4, dtypes.F32)
    assert e.value.code == npas.E_MASK_NOT_BLOCK_UNIFORM and "filter 1" in str(e.value)
    bad = m.copy()
    bad[0, 0, 0, 0] = 3
    with pytest.raises(npas.NpasError) as e:
        npas.pack_block_punched(w, bad, 4, 4, dtypes.F32)
    assert e.value.code == npas.E_MASK_VALUE
    mf = masks.fc_block_mask(32, 64, 16, 32, 4, 17)
    hole = mf.copy()
    hole[5, int(np.flatnonzero(mf[5])[0])] = 0
    with pytest.raises(npas.NpasError) as e:
        npas.pack_fc_block(np.zeros((32, 64), np.float32), hole, 16, 32, dtypes.F32)
    assert e.value.code == npas.E_MASK_NOT_BLOCK_UNIFORM
    lib = masks.pattern_library(8, 5)
    mp, _ = masks.pattern_mask(6, 6, lib, 0.3, 18)
    badp = mp.copy()
    k = np.argwhere(mp.reshape(36, 9).sum(1) == 4)[0, 0]
    badp.reshape(36, 9)[k, 4] = 0
    with pytest.raises(npas.NpasError) as e:
        npas.pack_pattern(np.zeros((6, 6, 3, 3), np.float32), badp, lib, dtypes.F32)
    assert e.value.code == npas.E_MASK_NOT_IN_LIBRARY
    with pytest.raises(npas.NpasError) as e:
        npas.pack_block_punched(w, m, 4, 4, 7)
    assert e.value.code == npas.E_DTYPE
    with pytest.raises(npas.NpasError) as e:
        npas.pack_block_punched(w, m, 0, 4, dtypes.F32)
    assert e.value.code == npas.E_SHAPE
    h = ctypes.c_void_p()
    assert npas.lib().npas_pack_block_punched(None, None, 1, 1, 1, 1, 1, 1, 0, None, ctypes.byref(h)) == npas.E_NULL


def test_run_calls_validate_arguments_before_touching_the_gpu():
    w = np.ones((4, 4, 3, 3), dtype=np.float32)
    p = npas.pack_block_punched(w, np.ones_like(w, dtype=np.uint8), 2, 2, dtypes.F32)
    L = npas.lib()
    assert L.npas_conv2d_sparse(p.handle, None, None, 1, 4, 4, 1, 1, None, None, 0, None) == npas.E_NULL
    assert L.npas_conv2d_sparse(p.handle, 256, 256, 0, 4, 4, 1, 1, None, None, 0, None) == npas.E_SHAPE
    assert L.npas_conv2d_sparse(p.handle, 256, 256, 1, 1, 1, 1, 0, None, None, 0, None) == npas.E_SHAPE   # empty output
    assert L.npas_fc_sparse(p.handle, 256, 256, 1, None, 0, None) == npas.E_SHAPE                          # 3x3 is no FC
    assert L.npas_maxpool3x3s2(None, None, 1, 4, 4, 4, 0, None) == npas.E_NULL
    assert L.npas_global_avgpool(256, 256, 1, 4, 4, 4, 9, None) == npas.E_DTYPE
    if not p.info()["device_ready"]:
        # no GPU here: the product path must fail loudly, never compute on the CPU
        assert L.npas_conv2d_sparse(p.handle, 256, 256, 1, 4, 4, 1, 1, None, None, 0, None) == npas.E_HIP
        assert "no device copy" in npas.last_error()


def test_stack_wiring_checks_and_workspace():
    w = configs.config5(batch=1, HW=32, width=16, blocks=(1, 1, 1, 1))
    packed = [helpers.pack_layer(npas, L, w.dtype) if L.kind in ("conv", "fc") else None for L in w.layers]
    descs = helpers.stack_descs(npas, w.layers, packed)
    st = npas.Stack(descs, 32, 32)
    assert st.num_launches() <= len(w.layers)
    ws1, ws4 = st.workspace_bytes(1), st.workspace_bytes(4)
    assert 0 < ws1 and ws1 % 256 == 0 and 3 * ws1 < ws4 <= 4 * ws1 + 256 * len(descs)
    # the workspace must at least hold the largest layer's live set: stem output + pooled output
    assert ws1 >= (16 * 16 * 16 + 8 * 8 * 16) * 2
    bad = [dict(d) for d in descs]
    bad[3]["src"] = 7                        # reads a tensor that does not exist yet
    with pytest.raises(npas.NpasError) as e:
        npas.Stack(bad, 32, 32)
    assert e.value.code == npas.E_SHAPE
    bad = [dict(d) for d in descs]
    bad[2]["res"] = 1                        # residual of the wrong shape
    with pytest.raises(npas.NpasError):
        npas.Stack(bad, 32, 32)
    assert npas.lib().npas_run_stack(st.handle, 256, 256, 1, None, 0, None) == npas.E_WORKSPACE


def _bp_layer(C, F, k, seed, rate=3):
    m = masks.block_punched_mask(F, C, k, k, 8, 4 if C % 4 == 0 else C, rate, seed)
    store, _ = dtypes.quantize(prng.normal(seed, 1, F * C * k * k, 0.1).reshape(F, C, k, k), dtypes.BF16)
    return npas.pack_block_punched(store, m, 8, 4 if C % 4 == 0 else C, dtypes.BF16)


def test_kernel_choice_follows_layer_and_launch_shape():
    """Host logic only: which kernel a layer gets depends on its shape and on how many tiles the launch has."""
    name = npas.conv2d_kernel_name
    p = _bp_layer(64, 64, 3, 41)                       # 3x3 on 64 channels, 64 filters: all weight stages fit in LDS
    assert name(p, 128, 56, 56, 1, 1) == "spatial_resident"
    assert name(p, 8, 56, 56, 1, 1) == "conv_slab_mfma"          # 112 tiles: too few for the persistent kernels
    assert name(p, 1, 56, 56, 1, 1) == "conv_smallm_mfma"        # little work in all: reduction split over the waves
    p = _bp_layer(128, 128, 3, 42)
    assert name(p, 128, 28, 28, 1, 1) == "spatial_ring"
    assert name(p, 128, 56, 56, 2, 1) == "spatial_ring"          # stride 2: phase planes
    assert name(p, 128, 56, 56, 2, 0) == "conv_slab_mfma"        # ... for pad 1 only
    assert name(p, 1, 28, 28, 1, 1) == "conv_smallm_mfma"
    p = _bp_layer(64, 256, 1, 43)
    assert name(p, 128, 56, 56, 1, 0) == "pointwise_ring"
    assert name(p, 1, 14, 14, 1, 0) == "conv_smallm_mfma"        # up to 256 output pixels
    assert name(p, 1, 56, 56, 1, 0) == "pointwise_ring"
    p = _bp_layer(1024, 256, 1, 46)
    assert name(p, 8, 7, 7, 1, 0) == "conv_smallm_mfma"          # long reduction, 7 x 16 workgroups: one round
    assert name(p, 32, 14, 14, 1, 0) == "pointwise_ring"
    p = _bp_layer(3, 64, 7, 44)
    assert name(p, 2, 224, 224, 2, 3) == "conv_smallc_mfma"      # fewer than 8 input channels
    p = _bp_layer(24, 144, 1, 45, rate=4)
    assert name(p, 64, 56, 56, 1, 0) == "conv_slab_mfma"         # channels not a multiple of 64


# ---- workspace placement of fused stacks (host logic: works without a GPU) -----------------------------------

def _pw(seed, idx, C, F, act, src, res=-1):
    return configs._bp_conv(seed, idx, C, F, 1, 1, 0, 8, 8, 2, 0.2, dtypes.BF16, act, src, res, name=f"pw{idx}")


def _dw(seed, idx, C, src, stride=1):
    ws, we = configs._tensor(seed, 150 + idx, (C, 3, 3), 0.3, dtypes.BF16)
    return configs.Layer("dwconv", "", C, C, 3, 3, stride, 1, 1, 1, 1.0, configs.ACT_RELU6, src, -1, ws, we, name=f"dw{idx}")


def _stack(layers, HW, flags):
    packed = [helpers.pack_layer(npas, L, dtypes.BF16) if L.kind in ("conv", "fc", "dwconv") else None for L in layers]
    return npas.Stack(helpers.stack_descs(npas, layers, packed), HW, HW, flags)


def _assert_placement_is_safe(st, N):
    """No launch may write over bytes that it, or a later launch, still has to read: tensors whose lifetimes
    (launch that writes them .. last launch that reads them) intersect must not share workspace bytes."""
    rows = st.describe(N)
    assert len(rows) == st.num_launches()
    born, last_read, where = {}, {}, {}
    for r, row in enumerate(rows):
        for key in ("src", "res"):
            t = row[key]
            if t >= 0:
                last_read[t] = r
                if row["off_" + key] >= 0:
                    assert where.setdefault(t, (row["off_" + key], row["bytes_" + key])) == (row["off_" + key], row["bytes_" + key])
        t = row["out"]
        born[t] = r
        if row["off_out"] >= 0:
            where[t] = (row["off_out"], row["bytes_out"])
            assert row["off_out"] % 256 == 0 and row["off_out"] + row["bytes_out"] <= st.workspace_bytes(N)
    ts = sorted(where)
    for i, a in enumerate(ts):
        for b in ts[i + 1:]:
            la, lb = (born.get(a, -1), last_read.get(a, born.get(a, -1))), (born.get(b, -1), last_read.get(b, born.get(b, -1)))
            if la[0] <= lb[1] and lb[0] <= la[1]:               # alive during a common launch
                (oa, sa), (ob, sb) = where[a], where[b]
                assert oa + sa <= ob or ob + sb <= oa, f"tensors {a} and {b} overlap in the workspace while both are alive"
    return rows


def test_fused_launches_never_write_over_their_own_inputs():
    A = configs
    # three fused 1x1 pairs in a row, of unequal widths (before the fix tensor 4 was placed over tensor 2)
    chain = [_pw(1, 0, 16, 48, A.ACT_RELU6, 0), _pw(1, 1, 48, 24, A.ACT_NONE, 1),
             _pw(1, 2, 24, 64, A.ACT_RELU6, 2), _pw(1, 3, 64, 8, A.ACT_NONE, 3),
             _pw(1, 4, 8, 40, A.ACT_RELU6, 4), _pw(1, 5, 40, 32, A.ACT_NONE, 5)]
    st = _stack(chain, 12, npas.STACK_FUSE_POINTWISE)
    rows = _assert_placement_is_safe(st, 3)
    assert [(r["first"], r["last"]) for r in rows] == [(0, 1), (2, 3), (4, 5)]
    assert rows[1]["off_src"] >= 0 and rows[1]["off_out"] >= 0
    # two inverted-residual blocks without residual, then a plain layer
    blocks = [_pw(2, 0, 16, 64, A.ACT_RELU6, 0), _dw(2, 1, 64, 1), _pw(2, 2, 64, 24, A.ACT_NONE, 2),
              _pw(2, 3, 24, 96, A.ACT_RELU6, 3), _dw(2, 4, 96, 4), _pw(2, 5, 96, 32, A.ACT_NONE, 5),
              _pw(2, 6, 32, 16, A.ACT_RELU, 6)]
    st = _stack(blocks, 10, npas.STACK_FUSE_INVERTED_RESIDUAL)
    rows = _assert_placement_is_safe(st, 2)
    assert [(r["first"], r["last"]) for r in rows] == [(0, 2), (3, 5), (6, 6)]
    # with a residual the fused block reads its input again at its last layer
    res = [_pw(3, 0, 24, 24, A.ACT_RELU, 0), _pw(3, 1, 24, 96, A.ACT_RELU6, 1), _dw(3, 2, 96, 2),
           _pw(3, 3, 96, 24, A.ACT_NONE, 3, res=1), _pw(3, 4, 24, 16, A.ACT_NONE, 4)]
    st = _stack(res, 9, npas.STACK_FUSE_INVERTED_RESIDUAL)
    rows = _assert_placement_is_safe(st, 2)
    assert (rows[1]["first"], rows[1]["last"], rows[1]["src"], rows[1]["res"]) == (1, 3, 1, 1)
    # the same stacks without fusion, and a residual stack with every fusion allowed
    for layers, hw in ((chain, 12), (blocks, 10), (res, 9)):
        _assert_placement_is_safe(_stack(layers, hw, 0), 2)
    w = configs.config5(batch=1, HW=32, width=16, blocks=(1, 2, 1, 1))
    for flags in (0, npas.STACK_FUSE_POINTWISE | npas.STACK_FUSE_INVERTED_RESIDUAL | npas.STACK_FUSE_CONV_MAXPOOL):
        st = _stack(w.layers, 32, flags)
        rows = _assert_placement_is_safe(st, 3)
        assert rows[-1]["off_out"] == -2 and rows[0]["off_src"] == -1


def test_a_layer_joins_one_fused_launch_only():
    """A 1x1 layer in front of a fused inverted-residual block must not swallow the block's first layer as the
    second half of a fused pair (the block would then never run)."""
    A = configs
    layers = [_pw(4, 0, 16, 24, A.ACT_RELU6, 0),
              _pw(4, 1, 24, 32, A.ACT_RELU6, 1), _dw(4, 2, 32, 2), _pw(4, 3, 32, 16, A.ACT_NONE, 3)]
    st = _stack(layers, 8, npas.STACK_FUSE_POINTWISE | npas.STACK_FUSE_INVERTED_RESIDUAL)
    rows = _assert_placement_is_safe(st, 2)
    assert [(r["first"], r["last"]) for r in rows] == [(0, 0), (1, 3)]
    assert {r["out"] for r in rows} == {1, 4}


def test_switches_are_read_once_and_can_be_replaced():
    p = _bp_layer(128, 128, 3, 42)
    assert npas.conv2d_kernel_name(p, 2, 14, 14, 1, 1) == "conv_smallm_mfma"
    npas.set_switches("spatial")
    try:
        assert npas.conv2d_kernel_name(p, 2, 14, 14, 1, 1) == "spatial_ring"
    finally:
        npas.set_switches(None)
    assert npas.conv2d_kernel_name(p, 2, 14, 14, 1, 1) == "conv_smallm_mfma"


def test_spatial_ring_is_not_planned_beyond_its_24_bit_pixel_count():
    """The spatial ring forms its patch addresses with 24-bit multiplies: a launch with 2^24 input pixels or more
    gets another kernel (the planner's rule, checked on the host)."""
    p = _bp_layer(128, 128, 3, 43)
    assert npas.conv2d_kernel_name(p, 128, 28, 28, 1, 1) == "spatial_ring"
    assert 21400 * 28 * 28 >= 1 << 24
    assert npas.conv2d_kernel_name(p, 21400, 28, 28, 1, 1) != "spatial_ring"
