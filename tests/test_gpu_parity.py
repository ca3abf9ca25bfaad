"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Packing metadata must be bit-exact; outputs
within max relative error 1e-2 (bf16) / 1e-5 (fp32), each layer fed the oracle's
rounded input (teacher forcing), stacks additionally end to end."""
import numpy as np
import pytest

import oracle
from tests import helpers
from tests.helpers import TOL, from_dev, new_dev, pack_layer, rel_err, run_layer_gpu, to_dev
from workloads import configs, dtypes, masks, prng

pytestmark = pytest.mark.gpu

# Stacks end to end: norm-wise bound on the final tensor (max |g - o| / max |o|) plus arg-max agreement.  Element-wise
# 1e-2 cannot hold through several roundings to bf16: a layer's fp32 and the oracle's fp64 sums can land on opposite
# sides of a rounding boundary of an intermediate value, which moves that value by a whole bf16 step (2^-8).
STACK_NORM_TOL = 1e-2


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "GPU tests need a GPU"
    return t


def layerwise(npas, torch, w, check_meta=True):
    """Teacher-forced layer-by-layer comparison of a workload; returns worst error."""
    rounded, raw = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    shapes = {0: w.x_shape}
    worst = 0.0
    for i, L in enumerate(w.layers):
        in_shape = shapes[L.src]
        shapes[i + 1] = helpers.out_shape(L, in_shape)
        packed = pack_layer(npas, L, w.dtype) if L.kind in ("conv", "fc", "dwconv") else None
        if packed is not None and check_meta and L.kind != "dwconv":
            helpers.check_metadata(oracle, L, packed, w.dtype)
            assert packed.info()["device_ready"] == 1
        xs, _ = dtypes.quantize(rounded[L.src], w.dtype)
        x_dev = to_dev(xs, torch)
        res_dev = None
        if L.res >= 0:
            rs, _ = dtypes.quantize(rounded[L.res], w.dtype)
            res_dev = to_dev(rs, torch)
        bias_dev = helpers.bias_tensors([L], torch)[0]
        y = run_layer_gpu(npas, torch, L, packed, x_dev, in_shape, w.dtype, res_dev, bias_dev)
        got = from_dev(y, w.dtype).reshape(shapes[i + 1])
        err = rel_err(got, rounded[i + 1].reshape(shapes[i + 1]))
        print(f"  layer {i:2d} {L.name or L.kind:12s} in={in_shape} out={shapes[i + 1]} err={err:.3e}", flush=True)
        assert err <= TOL[w.dtype], (i, L.name, err)
        worst = max(worst, err)
    return worst


def test_config1_conv3x3_fp32(npas, torch):
    print("config1 fp32 3x3", flush=True)
    w = configs.config1()
    p = pack_layer(npas, w.layers[0], w.dtype)
    assert npas.conv2d_kernel_name(p, 1, 32, 32, 1, 1) == "conv_wave_f32"      # reductions split over lanes
    layerwise(npas, torch, w)


def test_config1_conv3x3_fp32_one_lane_per_output(npas, torch, force_variant):
    force_variant("valu")
    w = configs.config1()
    p = pack_layer(npas, w.layers[0], w.dtype)
    assert npas.conv2d_kernel_name(p, 1, 32, 32, 1, 1) == "conv_valu_f32"
    layerwise(npas, torch, w)


WAVE_F32 = [
    ("wf_stride2_res_bias_hswish", 2, 9, 9, 8, 12, 3, 3, 2, 1, 4, 4, 2, dtypes.F32, 3, True, True),
    ("wf_wide_group_1x1", 1, 5, 5, 8, 24, 1, 1, 1, 0, 24, 8, 2, dtypes.F32, 0, False, False),
    ("wf_list_not_a_multiple_of_8", 3, 7, 6, 5, 6, 3, 3, 1, 1, 2, 5, 3, dtypes.F32, 1, False, True),
    ("wf_single_filter_groups", 1, 6, 6, 4, 5, 3, 3, 1, 1, 1, 1, 2, dtypes.F32, 2, True, False),
    ("wf_ragged_lanes", 1, 3, 5, 16, 8, 5, 5, 1, 2, 8, 4, 5, dtypes.F32, 0, False, True),
]


@pytest.mark.parametrize("case", WAVE_F32, ids=[c[0] for c in WAVE_F32])
def test_fp32_lane_split_kernel(npas, torch, case):
    _run_edge_case(npas, torch, case, expect_kernel="conv_wave_f32")


def test_config2_pointwise_stack_small(npas, torch):
    print("config2 small batch", flush=True)
    layerwise(npas, torch, configs.config2(batch=2, HW=23))        # 1058 pixels: several tiles + ragged tail


def test_config3_fc_block_full(npas, torch):
    print("config3 full", flush=True)
    w = configs.config3()
    p = pack_layer(npas, w.layers[0], w.dtype)
    assert npas.conv2d_kernel_name(p, w.x_shape[0], 1, 1, 1, 0) == "fc_gather_mfma"    # the exact-list kernel
    layerwise(npas, torch, w)


def test_config3_fc_block_full_dense_format_route(npas, torch, force_variant):
    """The same layer through the route that multiplies the dense weight images (what the exact-list kernel replaced)."""
    force_variant("nofcgather")
    w = configs.config3()
    p = pack_layer(npas, w.layers[0], w.dtype)
    assert npas.conv2d_kernel_name(p, w.x_shape[0], 1, 1, 1, 0) != "fc_gather_mfma"
    layerwise(npas, torch, w)


FC_GATHER = [
    # name, B (as N x H x W), C, F, stride, Bf, Bc, rate, dtype, act, use_res, use_bias
    ("fcg_ragged_rows_and_tiles", (37, 1, 1), 192, 88, 1, 16, 32, 5, dtypes.BF16, 1, False, True),
    ("fcg_one_row", (1, 1, 1), 64, 16, 1, 16, 32, 4, dtypes.BF16, 0, False, False),
    ("fcg_8x4_blocks_union_of_two_groups", (3, 9, 11), 256, 136, 1, 8, 4, 5, dtypes.BF16, 3, True, True),
    ("fcg_fp16_long_list", (5, 1, 1), 2048, 40, 1, 16, 32, 2.5, dtypes.F16, 2, False, True),
    ("fcg_strided_1x1", (3, 15, 14), 320, 72, 2, 8, 4, 5, dtypes.BF16, 2, True, False),
    ("fcg_many_tiles_two_rows", (2, 1, 1), 96, 1000, 1, 16, 32, 5, dtypes.BF16, 0, False, True),
]


@pytest.mark.parametrize("case", FC_GATHER, ids=[c[0] for c in FC_GATHER])
def test_fc_gather_kernel(npas, torch, case):
    name, (N, H, W), C, F, stride, Bf, Bc, rate, dtype, act, use_res, use_bias = case
    _run_edge_case(npas, torch, (name, N, H, W, C, F, 1, 1, stride, 0, Bf, Bc, rate, dtype, act, use_res, use_bias),
                   expect_kernel="fc_gather_mfma")


def test_config4_pattern_small(npas, torch):
    print("config4 small", flush=True)
    layerwise(npas, torch, configs.config4(batch=2, HW=28))


def test_config5_residual_stack_reduced(npas, torch):
    print("config5 reduced (64x64 input, width 16)", flush=True)
    layerwise(npas, torch, configs.config5(batch=2, HW=64, width=16))


def test_config5_full_size_batch1_layerwise(npas, torch):
    print("config5 full size, batch 1", flush=True)
    layerwise(npas, torch, configs.config5(batch=1), check_meta=False)


EDGE = [
    # name, N, H, W, C, F, KH, KW, stride, pad, Bf, Bc, rate, dtype, act, use_res, use_bias
    ("ragged_F_and_tail", 3, 9, 11, 16, 40, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 1, True, True),
    ("stem_like_C3_7x7s2", 2, 29, 31, 3, 24, 7, 7, 2, 3, 8, 4, 2, dtypes.BF16, 1, False, True),
    ("stride2_3x3_two_chunks", 2, 15, 14, 128, 72, 3, 3, 2, 1, 8, 4, 3, dtypes.BF16, 0, False, False),
    ("pointwise_stride2", 2, 15, 14, 320, 72, 1, 1, 2, 0, 8, 4, 5, dtypes.BF16, 2, False, False),
    ("unstructured_1x1_blocks", 1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 1, 3, dtypes.BF16, 0, False, False),
    ("coarse_whole_tensor_block", 1, 8, 8, 16, 32, 3, 3, 1, 1, 32, 16, 2, dtypes.BF16, 0, False, False),
    ("rate1_dense", 1, 6, 7, 8, 16, 3, 3, 1, 1, 8, 4, 1, dtypes.BF16, 0, False, False),
    ("one_pixel_input", 1, 1, 1, 64, 48, 1, 1, 1, 0, 8, 4, 2, dtypes.BF16, 0, False, False),
    ("fp16_storage", 2, 10, 10, 32, 32, 3, 3, 1, 1, 8, 4, 2, dtypes.F16, 1, True, False),
    ("fp32_stride2_res_bias", 2, 9, 9, 8, 12, 3, 3, 2, 1, 4, 4, 2, dtypes.F32, 2, True, True),
    ("fp32_wide_group", 1, 5, 5, 8, 24, 1, 1, 1, 0, 24, 8, 2, dtypes.F32, 0, False, False),
    ("large_C_many_chunks", 1, 7, 7, 600, 130, 1, 1, 1, 0, 8, 4, 2, dtypes.BF16, 1, True, False),
    ("kernel_5x3", 1, 30, 30, 8, 16, 5, 3, 1, 2, 4, 4, 2, dtypes.BF16, 0, False, False),
    # 100 items of 256 x 128 but 196 of 128 x 128: the pointwise ring's half-size tiles, ragged last tile
    ("pointwise_half_size_tiles", 127, 7, 7, 128, 512, 1, 1, 1, 0, 8, 4, 3, dtypes.BF16, 1, True, True),
    # pixel tiles evened out over the workgroups: 196 items of 256 pixels become 252 of 200 (the fourth
    # pixel group of a tile holds 8 pixels), and 100 of 256 become 200 of 128 (two pixel groups empty)
    ("pointwise_tiles_of_200_pixels", 1, 112, 112, 64, 512, 1, 1, 1, 0, 8, 4, 3, dtypes.BF16, 1, True, True),
    ("pointwise_tiles_of_128_pixels", 2, 80, 80, 64, 256, 1, 1, 1, 0, 8, 4, 2, dtypes.BF16, 2, True, False),
    # 50 items of 256 x 128: too few; 392 of 64 x 64 would take two rounds, 98 of 128 x 128 take one
    ("pointwise_medium_tiles_instead_of_small", 32, 14, 14, 256, 256, 1, 1, 1, 0, 8, 4, 3, dtypes.BF16, 1, False, True),
]


def _run_edge_case(npas, torch, case, expect_kernel=None):
    name, N, H, W, C, F, KH, KW, stride, pad, Bf, Bc, rate, dtype, act, use_res, use_bias = case
    print(f"edge {name}", flush=True)
    xs, xe = dtypes.quantize(prng.normal(7, 1, N * H * W * C).reshape(N, H, W, C), dtype)
    ws, we = dtypes.quantize(prng.normal(7, 2, F * C * KH * KW, 0.2).reshape(F, C, KH, KW), dtype)
    m = masks.block_punched_mask(F, C, KH, KW, Bf, Bc, rate, 99)
    L = configs.Layer("conv", "block_punched", C, F, KH, KW, stride, pad, Bf, Bc, rate, act, w_store=ws, w_exact=we, mask=m)
    oshape = helpers.out_shape(L, (N, H, W, C))
    bias = prng.normal(7, 3, F).astype(np.float32) if use_bias else None
    rs = re = None
    if use_res:
        rs, re = dtypes.quantize(prng.normal(7, 4, int(np.prod(oshape))).reshape(oshape), dtype)
    ref = oracle.round_to(oracle.conv2d_masked(xe, we, m, stride, pad, None if bias is None else bias.astype(np.float64),
                                               re, act), dtype)
    p = pack_layer(npas, L, dtype)
    helpers.check_metadata(oracle, L, p, dtype)
    if expect_kernel is not None:
        assert npas.conv2d_kernel_name(p, N, H, W, stride, pad) == expect_kernel
    y = run_layer_gpu(npas, torch, L, p, to_dev(xs, torch), (N, H, W, C), dtype,
                      None if rs is None else to_dev(rs, torch), None if bias is None else to_dev(bias, torch))
    got = from_dev(y, dtype).reshape(oshape)
    err = rel_err(got, ref)
    print(f"  err={err:.3e}", flush=True)
    assert err <= TOL[dtype]
    # run-to-run determinism: no atomics, one writer per element
    y2 = run_layer_gpu(npas, torch, L, p, to_dev(xs, torch), (N, H, W, C), dtype,
                       None if rs is None else to_dev(rs, torch), None if bias is None else to_dev(bias, torch))
    assert torch.equal(y, y2)


@pytest.mark.parametrize("case", EDGE, ids=[c[0] for c in EDGE])
def test_edge_cases(npas, torch, case):
    _run_edge_case(npas, torch, case)


# k x k, stride 1, whole 64-channel chunks: the streaming kernel (forced, so that small
# problems take it too): several images per tile, ragged tiles in every direction, filter
# counts off the 128-filter block, more work items than workgroups.
SPATIAL = [
    ("sp_7x7_images_per_tile", 11, 7, 7, 64, 136, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 1, True, True),
    ("sp_14x14_two_chunks", 3, 14, 14, 128, 64, 3, 3, 1, 1, 8, 4, 2, dtypes.BF16, 2, False, True),
    ("sp_ragged_tiles", 2, 30, 29, 64, 260, 3, 3, 1, 1, 4, 4, 2, dtypes.BF16, 0, True, False),
    ("sp_pad0_fp16", 2, 12, 12, 64, 32, 3, 3, 1, 0, 4, 4, 2, dtypes.F16, 1, False, False),
    ("sp_kernel_5x3", 2, 12, 17, 128, 32, 5, 3, 1, 2, 4, 4, 2, dtypes.BF16, 0, False, False),
    ("sp_more_items_than_workgroups", 70, 16, 16, 64, 512, 3, 3, 1, 1, 8, 4, 4, dtypes.BF16, 1, True, True),
]


@pytest.mark.parametrize("case", SPATIAL, ids=[c[0] for c in SPATIAL])
def test_spatial_streaming_kernel(npas, torch, case, force_variant):
    force_variant("spatial")
    _run_edge_case(npas, torch, case, expect_kernel="spatial_ring")


RESIDENT = [
    ("res_3x3_64", 3, 20, 23, 64, 64, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 1, True, True),
    ("res_ragged_filters_fp16", 2, 13, 11, 64, 40, 3, 3, 1, 1, 8, 4, 2, dtypes.F16, 2, False, True),
    ("res_two_chunks_2x2_pad0", 5, 9, 9, 128, 32, 2, 2, 1, 0, 4, 4, 2, dtypes.BF16, 0, True, False),
    ("res_several_images_per_tile", 37, 7, 7, 64, 64, 3, 3, 1, 1, 8, 4, 5, dtypes.BF16, 1, False, False),
    ("res_more_items_than_workgroups", 20, 56, 56, 64, 16, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 1, False, True),
]


@pytest.mark.parametrize("case", RESIDENT, ids=[c[0] for c in RESIDENT])
def test_spatial_resident_weights_kernel(npas, torch, case, force_variant):
    force_variant("resident")
    _run_edge_case(npas, torch, case, expect_kernel="spatial_resident")


def test_spatial_resident_weights_kernel_chosen_for_a_full_launch(npas, torch):
    """56 x 56, 64 -> 64 at batch 16: 224 tiles of 8 x 28 pixels, chosen by the library itself."""
    _run_edge_case(npas, torch, ("res_full_launch", 16, 56, 56, 64, 64, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 1, False, True),
                   expect_kernel="spatial_resident")


SPATIAL_STRIDE2 = [
    ("sp2_ragged", 3, 17, 19, 64, 128, 3, 3, 2, 1, 8, 4, 3, dtypes.BF16, 1, True, True),
    ("sp2_two_chunks_fp16", 2, 24, 24, 128, 72, 3, 3, 2, 1, 8, 4, 2, dtypes.F16, 2, False, True),
    ("sp2_several_images_per_tile", 21, 14, 14, 64, 64, 3, 3, 2, 1, 8, 4, 5, dtypes.BF16, 0, True, False),
    ("sp2_even_input_one_row_tiles", 2, 6, 40, 64, 32, 3, 3, 2, 1, 4, 4, 2, dtypes.BF16, 1, False, False),
    ("sp2_more_items_than_workgroups", 70, 32, 32, 64, 512, 3, 3, 2, 1, 8, 4, 4, dtypes.BF16, 1, False, True),
]


@pytest.mark.parametrize("case", SPATIAL_STRIDE2, ids=[c[0] for c in SPATIAL_STRIDE2])
def test_spatial_streaming_kernel_stride2(npas, torch, case, force_variant):
    force_variant("spatial")
    _run_edge_case(npas, torch, case, expect_kernel="spatial_ring")


def test_spatial_streaming_kernel_half_size_tiles(npas, torch):
    """104 tiles of 256 pixels would leave most CUs idle; 256 tiles of 128 pixels (two 7x7 images each) do not:
    the streaming kernel with half the multiplying waves, chosen by the library itself."""
    _run_edge_case(npas, torch, ("sp_7x7_half_tiles", 128, 7, 7, 64, 512, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 1, True, True),
                   expect_kernel="spatial_ring")


def test_config4_pattern_small_streaming_kernel(npas, torch, force_variant):
    force_variant("spatial")
    print("config4 small, streaming kernel", flush=True)
    layerwise(npas, torch, configs.config4(batch=3, HW=12))


SWEEP_CASES = [(sch, r) for sch in ("block_punched", "unstructured", "whole_tensor", "pattern", "filter")
               for r in (2.5, 10) if not (sch == "pattern" and r < 2.25)]


@pytest.mark.parametrize("scheme,rate", SWEEP_CASES, ids=["%s_r%s" % c for c in SWEEP_CASES])
def test_rate_sweep_layer_kinds(npas, torch, scheme, rate):
    """The layer kinds of the rate sweep (bench.py --sweep rate), at a size the oracle finishes quickly."""
    from workloads import sweeps
    print(f"sweep {scheme} rate {rate}", flush=True)
    layerwise(npas, torch, sweeps.rate_sweep_layer(scheme, rate, batch=2, HW=11, C=64, F=72))


def test_block_sweep_stack_reduced(npas, torch):
    """The block-size sweep's stack (bench.py --sweep block) at 16x8 blocks, reduced input size."""
    from workloads import sweeps
    print("block sweep 16x8", flush=True)
    layerwise(npas, torch, sweeps.block_sweep_stack(16, 8, batch=1, HW=32), check_meta=False)


DW_CASES = [
    # name, N, H, W, C, stride, dtype, act, use_res, use_bias
    ("dw_bf16_vec", 2, 13, 11, 144, 1, dtypes.BF16, 2, False, True),
    ("dw_bf16_stride2_odd", 3, 15, 14, 24, 2, dtypes.BF16, 2, False, False),
    ("dw_bf16_scalar_channels", 1, 9, 9, 12, 1, dtypes.BF16, 1, True, True),
    ("dw_fp16_res", 2, 8, 10, 32, 1, dtypes.F16, 0, True, False),
    ("dw_fp32", 1, 7, 8, 10, 2, dtypes.F32, 2, True, True),
    ("dw_one_pixel", 1, 1, 1, 16, 1, dtypes.BF16, 0, False, False),
    ("dw_bf16_hardswish", 2, 13, 11, 40, 1, dtypes.BF16, 3, True, True),
    ("dw_fp32_hardswish_scalar", 1, 6, 7, 5, 1, dtypes.F32, 3, False, True),
]


@pytest.mark.parametrize("case", DW_CASES, ids=[c[0] for c in DW_CASES])
def test_depthwise3x3(npas, torch, case):
    name, N, H, W, C, stride, dtype, act, use_res, use_bias = case
    print(f"depthwise {name}", flush=True)
    xs, xe = dtypes.quantize(prng.normal(17, 1, N * H * W * C).reshape(N, H, W, C), dtype)
    ws, we = dtypes.quantize(prng.normal(17, 2, C * 9, 0.3).reshape(C, 3, 3), dtype)
    L = configs.Layer("dwconv", "", C, C, 3, 3, stride, 1, 1, 1, 1.0, act, w_store=ws, w_exact=we)
    oshape = helpers.out_shape(L, (N, H, W, C))
    bias = prng.normal(17, 3, C).astype(np.float32) if use_bias else None
    rs = re = None
    if use_res:
        rs, re = dtypes.quantize(prng.normal(17, 4, int(np.prod(oshape))).reshape(oshape), dtype)
    ref = oracle.round_to(oracle.dwconv3x3(xe, we, stride, None if bias is None else bias.astype(np.float64), re, act), dtype)
    p = pack_layer(npas, L, dtype)
    info = p.info()
    assert info["scheme"] == npas.SCHEME_DEPTHWISE and info["C"] == C and info["device_ready"] == 1
    np.testing.assert_array_equal(p.export()["w_compact"], np.asarray(ws).reshape(C, 9))    # bit-exact round trip
    y = run_layer_gpu(npas, torch, L, p, to_dev(xs, torch), (N, H, W, C), dtype,
                      None if rs is None else to_dev(rs, torch), None if bias is None else to_dev(bias, torch))
    err = rel_err(from_dev(y, dtype).reshape(oshape), ref)
    print(f"  err={err:.3e}", flush=True)
    assert err <= TOL[dtype]


@pytest.mark.parametrize("stride,bias,act,HW", [(1, False, configs.ACT_RELU6, 13), (2, False, configs.ACT_RELU6, 13),
                                                (1, True, configs.ACT_RELU6, 13), (2, True, configs.ACT_RELU6, 13),
                                                (2, True, configs.ACT_HARDSWISH, 14), (1, True, configs.ACT_HARDSWISH, 9),
                                                (2, False, configs.ACT_RELU6, 31)],
                         ids=["s1", "s2", "s1_bias", "s2_bias", "s2_bias_hswish_even", "s1_bias_hswish", "s2_several_tiles"])
def test_inverted_residual_block_layerwise_and_stack(npas, torch, stride, bias, act, HW):
    """1x1 -> depthwise 3x3 (stride 1 or 2) -> 1x1 (+ input at stride 1), with and without a bias per layer: each layer
    against the oracle, then the stack call end to end, per layer and as one fused launch.  With a bias the padding
    of the depthwise layer must still be zero (not act(bias)): the border pixels are where that shows."""
    from workloads import sweeps
    w = sweeps.inverted_residual_block(batch=2, HW=HW, stride=stride, bias=bias, act=act)
    print(f"inverted residual block, stride {stride} bias {bias} act {act} {HW}x{HW}", flush=True)
    layerwise(npas, torch, w)
    rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    for flags in (0, 1, 3):          # per layer; pointwise-pair fusion (not applicable); whole-block fusion
        got, st = _run_stack_gpu(npas, torch, w, flags)
        assert st.num_launches() == (1 if flags == 3 else 3)
        norm, worst = helpers.check_stack_output(got, rounded[-1], STACK_NORM_TOL)
        print(f"  run_stack flags={flags} launches={st.num_launches()} norm-wise {norm:.3e} worst element {worst:.3e}", flush=True)
        border = np.concatenate([got[:, 0].ravel(), got[:, -1].ravel(), got[:, :, 0].ravel(), got[:, :, -1].ravel()])
        want = np.concatenate([rounded[-1][:, 0].ravel(), rounded[-1][:, -1].ravel(), rounded[-1][:, :, 0].ravel(), rounded[-1][:, :, -1].ravel()])
        assert rel_err(border, want) <= 0.1, "border pixels (padding of the depthwise layer)"


def test_run_stack_in_a_hip_graph_replays_like_the_eager_call(npas, torch):
    """npas_run_stack allocates nothing and clears nothing during a run, so a caller may capture it.
    Several replays, with eager work and synchronisations in between, each against the eager result."""
    print("run_stack captured in a HIP graph", flush=True)
    w = configs.config5(batch=2, HW=32, width=16, blocks=(1, 1, 1, 1))
    packed = [pack_layer(npas, L, w.dtype) if L.kind in ("conv", "fc", "dwconv") else None for L in w.layers]
    st = npas.Stack(helpers.stack_descs(npas, w.layers, packed), w.x_shape[1], w.x_shape[2],
                    npas.STACK_FUSE_POINTWISE | npas.STACK_FUSE_INVERTED_RESIDUAL | npas.STACK_FUSE_CONV_MAXPOOL)
    N = w.x_shape[0]
    shapes = {0: w.x_shape}
    for i, L in enumerate(w.layers):
        shapes[i + 1] = helpers.out_shape(L, shapes[L.src])
    wsb = st.workspace_bytes(N)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    x = to_dev(w.x_store, torch)
    y_eager = new_dev(shapes[len(w.layers)], w.dtype, torch, fill=0x7FC1)
    st.run(x, y_eager, N, ws, wsb)           # also the first call: one-time kernel attributes are set here
    torch.cuda.synchronize()
    y_graph = new_dev(shapes[len(w.layers)], w.dtype, torch, fill=0x7FC1)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        st.run(x, y_graph, N, ws, wsb, torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        y_graph.fill_(0x7FC1)                # eager work between the replays
        ws.random_(0, 255)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), f"replay {rep} differs from the eager call"


def test_depthwise_handle_is_rejected_by_the_convolution_call(npas, torch):
    ws, _ = dtypes.quantize(prng.normal(18, 1, 16 * 9).reshape(16, 3, 3), dtypes.BF16)
    p = npas.pack_depthwise3x3(ws, dtypes.BF16)
    x = new_dev((1, 4, 4, 16), dtypes.BF16, torch, fill=0)
    y = new_dev((1, 4, 4, 16), dtypes.BF16, torch, fill=0)
    with pytest.raises(npas.NpasError):
        npas.conv2d_sparse(p, x, y, 1, 4, 4, 1, 1)


def test_fc_with_rows_and_columns_pruned_inside_blocks(npas, torch):
    """Block-based FC pruning allows whole rows as well as whole columns of a block to go (section 3)."""
    B, IN, OUT, Br, Bcol = 37, 192, 88, 16, 32
    m = masks.fc_block_mask(OUT, IN, Br, Bcol, 3, 41).copy()
    keys = prng.u64(41, 9, OUT * (IN // Bcol)).reshape(OUT, IN // Bcol)
    rowdrop = (keys % np.uint64(4)) == 0                      # a quarter of the (row, block) pairs lose their row
    m[np.repeat(rowdrop, Bcol, axis=1)] = 0
    assert oracle.validate_fc_block(m, Br, Bcol) == 0
    xs, xe = dtypes.quantize(prng.normal(41, 1, B * IN).reshape(B, IN), dtypes.BF16)
    ws, we = dtypes.quantize(prng.normal(41, 2, OUT * IN, 0.1).reshape(OUT, IN, 1, 1), dtypes.BF16)
    L = configs.Layer("fc", "fc_block", IN, OUT, 1, 1, 1, 0, Br, Bcol, 3.0, 1, w_store=ws, w_exact=we,
                      mask=m.reshape(OUT, IN, 1, 1))
    p = pack_layer(npas, L, dtypes.BF16)
    helpers.check_metadata(oracle, L, p, dtypes.BF16)
    y = run_layer_gpu(npas, torch, L, p, to_dev(xs, torch), (B, IN), dtypes.BF16)
    ref = oracle.round_to(oracle.fc_masked(xe, we, L.mask, None, 1), dtypes.BF16)
    err = rel_err(from_dev(y, dtypes.BF16).reshape(B, OUT), ref)
    print(f"  err={err:.3e}", flush=True)
    assert err <= 1e-2


# Fewer than 8 input channels (an image stem): the whole-reduction kernel.  Ragged tiles, stride 2 with
# padding 3, one to five reduction steps, filter counts below 64, more tiles than workgroups.
SMALLC = [
    ("stem_7x7_s2", 2, 37, 41, 3, 64, 7, 7, 2, 3, 8, 3, 3, dtypes.BF16, 1, False, True),
    ("c1_3x3_f16", 3, 19, 23, 1, 16, 3, 3, 1, 1, 4, 1, 2, dtypes.F16, 1, True, True),
    ("c4_5x5_f36", 2, 20, 18, 4, 36, 5, 5, 1, 2, 4, 4, 2, dtypes.BF16, 2, True, False),
    ("c3_3x3_s2_f8", 1, 9, 9, 3, 8, 3, 3, 2, 1, 8, 3, 2, dtypes.BF16, 0, False, False),
    ("c3_3x3_many_tiles", 13, 128, 128, 3, 8, 3, 3, 1, 1, 8, 3, 2, dtypes.BF16, 1, False, True),
]


@pytest.mark.parametrize("case", SMALLC, ids=[c[0] for c in SMALLC])
def test_small_channel_kernel(npas, torch, case):
    _run_edge_case(npas, torch, case, expect_kernel="conv_smallc_mfma")


# Few output pixels (batch 1, late stages): the kernel that splits the reduction over the waves of a workgroup.
# Stride 2, non-square kernels, filter counts off the 16- and 128-filter grids, ragged pixel tiles, fp16.
SMALLM = [
    ("sm_7x7_512", 1, 7, 7, 512, 512, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 1, False, True),
    ("sm_stride2_ragged", 3, 15, 14, 128, 72, 3, 3, 2, 1, 8, 4, 3, dtypes.BF16, 0, True, True),
    ("sm_5x3_fp16", 2, 12, 17, 64, 200, 5, 3, 1, 2, 4, 4, 2, dtypes.F16, 2, True, False),
    ("sm_one_step_per_wave", 1, 9, 9, 64, 64, 3, 3, 1, 1, 8, 4, 2, dtypes.BF16, 1, False, False),
    ("sm_more_waves_than_steps", 1, 5, 5, 64, 40, 2, 2, 1, 0, 8, 4, 2, dtypes.BF16, 0, False, False),
    ("sm_many_pixels_little_work", 1, 41, 39, 64, 64, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 1, True, True),
]


@pytest.mark.parametrize("case", SMALLM, ids=[c[0] for c in SMALLM])
def test_small_pixel_count_kernel(npas, torch, case):
    _run_edge_case(npas, torch, case, expect_kernel="conv_smallm_mfma")


def test_block_punched_5x5(npas, torch):
    _run_edge_case(npas, torch, ("kernel_5x5", 2, 17, 19, 16, 24, 5, 5, 1, 2, 8, 4, 3, dtypes.BF16, 1, False, True))
    _run_edge_case(npas, torch, ("kernel_5x5_wide", 2, 12, 12, 64, 72, 5, 5, 1, 2, 8, 4, 2, dtypes.BF16, 0, True, False))


def test_group_with_everything_pruned_gives_bias_only(npas, torch):
    F, C = 32, 16
    m = masks.block_punched_mask(F, C, 3, 3, 8, 4, 2, 5)
    m[8:16] = 0                                  # filter group 1 keeps nothing
    ws, we = dtypes.quantize(prng.normal(8, 2, F * C * 9, 0.2).reshape(F, C, 3, 3), dtypes.BF16)
    xs, xe = dtypes.quantize(prng.normal(8, 1, 6 * 6 * C).reshape(1, 6, 6, C), dtypes.BF16)
    bias = prng.normal(8, 3, F).astype(np.float32)
    L = configs.Layer("conv", "block_punched", C, F, 3, 3, 1, 1, 8, 4, 2, 0, w_store=ws, w_exact=we, mask=m)
    p = pack_layer(npas, L, dtypes.BF16)
    y = from_dev(run_layer_gpu(npas, torch, L, p, to_dev(xs, torch), (1, 6, 6, C), dtypes.BF16, None, to_dev(bias, torch)),
                 dtypes.BF16).reshape(1, 6, 6, F)
    ref = oracle.round_to(oracle.conv2d_masked(xe, we, m, 1, 1, bias.astype(np.float64)), dtypes.BF16)
    np.testing.assert_array_equal(y[..., 8:16], ref[..., 8:16])
    assert rel_err(y, ref) <= 1e-2


def test_garbage_under_the_mask_changes_nothing(npas, torch):
    w = configs.config2(batch=1, HW=9)
    L = w.layers[0]
    junk = L.w_store.copy()
    junk[L.mask == 0] = 0x7F80                    # +inf bit pattern where pruned
    p1 = npas.pack_block_punched(L.w_store, L.mask, L.Bf, L.Bc, w.dtype)
    p2 = npas.pack_block_punched(junk, L.mask, L.Bf, L.Bc, w.dtype)
    x = to_dev(w.x_store, torch)
    y1 = run_layer_gpu(npas, torch, L, p1, x, w.x_shape, w.dtype)
    y2 = run_layer_gpu(npas, torch, L, p2, x, w.x_shape, w.dtype)
    assert torch.equal(y1, y2)


def _run_stack_gpu(npas, torch, w, flags=0):
    packed = [pack_layer(npas, L, w.dtype) if L.kind in ("conv", "fc", "dwconv") else None for L in w.layers]
    biases = helpers.bias_tensors(w.layers, torch)   # alive until the run below has finished
    st = npas.Stack(helpers.stack_descs(npas, w.layers, packed, biases), w.x_shape[1], w.x_shape[2], flags)
    N = w.x_shape[0]
    shape = w.x_shape
    shapes = {0: shape}
    for i, L in enumerate(w.layers):
        shapes[i + 1] = helpers.out_shape(L, shapes[L.src])
    wsb = st.workspace_bytes(N)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    y = new_dev(shapes[len(w.layers)], w.dtype, torch, fill=(float("nan") if w.dtype == dtypes.F32 else 0x7FC1))
    st.run(to_dev(w.x_store, torch), y, N, ws, wsb)
    torch.cuda.synchronize()
    return from_dev(y, w.dtype).reshape(shapes[len(w.layers)]), st


@pytest.mark.parametrize("flags", [0, 1], ids=["per_layer", "fused_pointwise"])
def test_config2_run_stack_end_to_end(npas, torch, flags):
    print(f"config2 run_stack flags={flags}", flush=True)
    w = configs.config2(batch=2, HW=23)
    got, st = _run_stack_gpu(npas, torch, w, flags)
    rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    err = rel_err(got, rounded[-1])
    print(f"  launches={st.num_launches()} err={err:.3e}", flush=True)
    assert err <= 1e-2


def test_fp16_storage_through_the_fused_kernels_and_the_pointwise_ring(npas, torch):
    """Every 16-bit kernel is instantiated for fp16 as well as bf16: the fused pair, the fused inverted-residual
    block and the streaming 1x1 kernel on fp16 tensors (fused launches: the stack criterion at the fp16 tolerance)."""
    from workloads import sweeps
    print("fp16: fused pair", flush=True)
    w = configs.config2(batch=2, HW=23, dtype=dtypes.F16)
    got, st = _run_stack_gpu(npas, torch, w, 1)
    rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    norm, worst = helpers.check_stack_output(got, rounded[-1], TOL[dtypes.F16])
    print(f"  launches={st.num_launches()} norm-wise {norm:.3e} worst element {worst:.3e}", flush=True)
    assert st.num_launches() == 1
    print("fp16: fused inverted-residual block", flush=True)
    w = sweeps.inverted_residual_block(batch=2, HW=13, dtype=dtypes.F16)
    got, st = _run_stack_gpu(npas, torch, w, 3)
    rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    norm, worst = helpers.check_stack_output(got, rounded[-1], TOL[dtypes.F16])
    print(f"  launches={st.num_launches()} norm-wise {norm:.3e} worst element {worst:.3e}", flush=True)
    assert st.num_launches() == 1
    _run_edge_case(npas, torch, ("fp16_pointwise_ring", 3, 9, 11, 128, 136, 1, 1, 1, 0, 8, 4, 3, dtypes.F16, 2, True, True),
                   expect_kernel="pointwise_ring")


def test_config5_run_stack_end_to_end(npas, torch):
    print("config5 reduced run_stack", flush=True)
    w = configs.config5(batch=2, HW=64, width=16)
    got, st = _run_stack_gpu(npas, torch, w, npas.STACK_FUSE_CONV_MAXPOOL)
    rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    ref = rounded[-1]
    norm_err = np.abs(got - ref).max() / np.abs(ref).max()
    print(f"  launches={st.num_launches()} norm-wise err={norm_err:.3e} elementwise={rel_err(got, ref):.3e}", flush=True)
    # 50+ bf16 layers: element-wise 1e-2 cannot hold end to end (roundings compound), the norm-wise bound must
    assert norm_err <= STACK_NORM_TOL
    assert (got.argmax(1) == ref.argmax(1)).all()


STEM_POOL = [
    # name, N, H, W, C, F, k, stride, pad, block channels, act, dtype
    ("stem7x7_ragged", 3, 37, 41, 3, 64, 7, 2, 3, 3, configs.ACT_RELU, dtypes.BF16),
    ("stem7x7_no_activation_fp16", 2, 64, 64, 3, 40, 7, 2, 3, 3, configs.ACT_NONE, dtypes.F16),
    ("conv3x3_stride1_4_channels", 2, 30, 33, 4, 32, 3, 1, 1, 4, configs.ACT_RELU6, dtypes.BF16),
    ("more_tiles_than_workgroups", 9, 224, 224, 3, 64, 7, 2, 3, 3, configs.ACT_RELU, dtypes.BF16),
]


@pytest.mark.parametrize("case", STEM_POOL, ids=[c[0] for c in STEM_POOL])
def test_conv_and_maxpool_as_one_kernel(npas, torch, case):
    """A small-channel conv and the 3x3 / stride 2 max pool after it, one launch (NPAS_STACK_FUSE_CONV_MAXPOOL): the
    pooled tensor against the oracle's conv -> round -> max pool, and against the two-launch stack bit for bit."""
    name, N, H, W, C, F, k, stride, pad, Bc, act, dtype = case
    print(f"conv+maxpool {name}", flush=True)
    xs, xe = configs._tensor(77, 1, (N, H, W, C), 1.0, dtype)
    layers = [configs._bp_conv(77, 0, C, F, k, stride, pad, 8, Bc, 2, 0.2, dtype, act, 0, -1, "stem"),
              configs.Layer("maxpool", src=1, C=F, F=F, KH=3, KW=3, stride=2, pad=1, name="maxpool")]
    w = configs.Workload("stem_pool", dtype, (N, H, W, C), xs, xe, layers)
    fused, st = _run_stack_gpu(npas, torch, w, npas.STACK_FUSE_CONV_MAXPOOL)
    plain, st0 = _run_stack_gpu(npas, torch, w, 0)
    assert st.num_launches() == 1 and st0.num_launches() == 2
    assert st.workspace_bytes(N) == 0
    np.testing.assert_array_equal(fused, plain)
    if N * H * W <= 64 * 64 * 4:
        rounded, _ = oracle.run_stack(xe, layers, dtype)
        err = rel_err(fused, rounded[-1])
        print(f"  err={err:.3e}", flush=True)
        assert err <= TOL[dtype]


def test_full_size_config2_two_launches_sampled(npas, torch):
    """configs[1] at full size (batch 64, 56x56) through npas_run_stack WITHOUT fusion (two launches of the per-layer
    kernel): sampled pixels against the oracle.  The fused launch is covered by the tests below."""
    print("config2 full size, two launches, sampled", flush=True)
    w = configs.config2()
    got, _ = _run_stack_gpu(npas, torch, w)
    N, H, W, C = w.x_shape
    npx = N * H * W
    idx = (prng.u64(3, 3, 4096) % np.uint64(npx)).astype(np.int64)
    idx[:8] = [0, 1, npx - 1, npx - 2, 127, 128, 129, npx // 2]
    xsub = w.x_exact.reshape(npx, C)[idx].reshape(1, 1, -1, C)
    rounded, _ = oracle.run_stack(xsub, w.layers, w.dtype)
    L2 = w.layers[1]
    err, beyond = helpers.check_two_layer_pointwise(got.reshape(npx, -1)[idx], rounded[-1].reshape(len(idx), -1), rounded[1],
                                                    (L2.w_exact * L2.mask).reshape(L2.F, L2.C))
    print(f"  worst plain err={err:.3e}, share beyond 1e-2: {beyond:.2e}", flush=True)


def _pixel_stack(M, dtype=dtypes.BF16):
    """configs[1]'s two layers on M pixels (a 1 x M image: every pixel of a 1x1 stack is independent)."""
    w = configs.config2(batch=1, HW=1, dtype=dtype)
    xs, xe = configs._tensor(configs.BASE_SEED + 2, 1, (1, 1, M, w.layers[0].C), 1.0, dtype)
    return configs.Workload("cfg2_pixels_%d" % M, dtype, (1, 1, M, w.layers[0].C), xs, xe, w.layers)


# 16-pixel blocks per wave of the fused pair: the kernel is instantiated per count (1..8) and a launch uses two
# neighbouring counts.  M pixels -> ceil(M / 16) blocks over min(ceil(blocks / 4), 512) (or more) workgroups x 4 waves.
FPP_COUNTS = [
    # M, grid, counts in use
    (16 * 5000 - 5, 512, {2, 3}),      # ragged last block
    (16 * 9000 - 10, 512, {4, 5}),
    (64 * 56 * 56, 512, {6, 7}),       # the benchmark's shape
    (16 * 16000 - 7, 512, {7, 8}),
    (16 * 20000, 625, {8}),            # more than 8 blocks per wave at 512 workgroups: the grid grows instead
    (16 * 2048 * 3 + 1, 512, {3, 4}),  # one pixel past a whole number of rounds
]


@pytest.mark.parametrize("M,grid,counts", FPP_COUNTS, ids=["cnt" + "_".join(map(str, sorted(c[2]))) + "_M%d" % c[0] for c in FPP_COUNTS])
def test_fused_pair_every_blocks_per_wave_instantiation(npas, torch, M, grid, counts):
    """Every pixel of the fused 1x1 -> ReLU6 -> 1x1 launch against the oracle, at pixel counts that put 2 .. 8
    blocks on a wave (the host formula for the split is restated here to make sure the case is what it claims)."""
    nblk = -(-M // 16)
    g = max(-(-nblk // 32), min(-(-nblk // 4), 512))
    base, extra = divmod(nblk, 4 * g)
    assert g == grid and ({base, base + 1} if extra else {base}) == counts
    print(f"fused pair M={M} blocks={nblk} grid={g} blocks per wave={sorted(counts)}", flush=True)
    w = _pixel_stack(M)
    got, st = _run_stack_gpu(npas, torch, w, npas.STACK_FUSE_POINTWISE)
    assert st.num_launches() == 1 and st.workspace_bytes(1) == 0
    rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    L2 = w.layers[1]
    err, beyond = helpers.check_two_layer_pointwise(got, rounded[-1], rounded[1], (L2.w_exact * L2.mask).reshape(L2.F, L2.C))
    print(f"  worst plain err={err:.3e}, share beyond 1e-2: {beyond:.2e}", flush=True)


def test_config2_benchmark_configuration_fused(npas, torch):
    """configs[1] exactly as bench.py times it (batch 64, 56 x 56, npas_run_stack with NPAS_STACK_FUSE_POINTWISE, one
    launch, waves of 6 and 7 blocks): every output pixel against the oracle, and the run repeated bit for bit."""
    print("config2 full size, fused, all pixels", flush=True)
    w = configs.config2()
    got, st = _run_stack_gpu(npas, torch, w, npas.STACK_FUSE_POINTWISE)
    assert st.num_launches() == 1
    rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    L2 = w.layers[1]
    err, beyond = helpers.check_two_layer_pointwise(got, rounded[-1], rounded[1], (L2.w_exact * L2.mask).reshape(L2.F, L2.C))
    print(f"  worst plain err={err:.3e}, share beyond 1e-2: {beyond:.2e}", flush=True)
    # first and last block of a few waves, separately (what a wrong block range would hit first)
    npx = got.shape[0] * got.shape[1] * got.shape[2]
    nblk = npx // 16
    base, extra = divmod(nblk, 2048)
    for gw in (0, 1, extra - 1, extra, extra + 1, 2047):
        b0 = gw * base + min(gw, extra)
        cnt = base + (1 if gw < extra else 0)
        for blk in (b0, b0 + cnt - 1):
            sl = slice(16 * blk, 16 * blk + 16)
            assert rel_err(got.reshape(npx, -1)[sl], rounded[-1].reshape(npx, -1)[sl]) <= 3e-2, (gw, blk)
    again, _ = _run_stack_gpu(npas, torch, w, npas.STACK_FUSE_POINTWISE)
    np.testing.assert_array_equal(got, again)


FULL_FLAGS = [0, 7]


@pytest.mark.parametrize("flags", FULL_FLAGS, ids=["per_layer", "all_fusions"])
def test_config5_full_size_run_stack_batch2_logits(npas, torch, flags):
    """The 50-layer stack at full size (224 x 224, all 53 pruned convs + pools + classifier) through npas_run_stack,
    two images, with no fusion and with every fusion flag bench.py sets: the logits against the oracle's
    (norm-wise, the bound stated for stacks end to end, and the arg-max)."""
    print(f"config5 full size run_stack batch 2 flags={flags}", flush=True)
    w = configs.config5(batch=2)
    got, st = _run_stack_gpu(npas, torch, w, flags)
    rounded, _ = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    ref = rounded[-1]
    norm_err = np.abs(got - ref).max() / np.abs(ref).max()
    print(f"  launches={st.num_launches()} norm-wise err={norm_err:.3e} elementwise={rel_err(got, ref):.3e}", flush=True)
    assert st.num_launches() == (len(w.layers) - 1 if flags else len(w.layers))
    assert norm_err <= STACK_NORM_TOL
    assert (got.argmax(1) == ref.argmax(1)).all()


def test_chained_fused_launches_against_the_oracle(npas, torch):
    """Fused launches whose inputs and outputs are workspace tensors (the placement must keep a fused launch's input
    alive while it writes the output of the last layer it absorbs): three fused 1x1 pairs of unequal widths in a row,
    and two fused inverted-residual blocks without residual, end to end against the oracle and against the
    unfused stack."""
    A = configs

    def pw(seed, idx, C, F, act, src, res=-1):
        return configs._bp_conv(seed, idx, C, F, 1, 1, 0, 8, 8, 2, 0.25, dtypes.BF16, act, src, res, name=f"pw{idx}")

    def dw(seed, idx, C, src):
        ws, we = configs._tensor(seed, 150 + idx, (C, 3, 3), 0.3, dtypes.BF16)
        return configs.Layer("dwconv", "", C, C, 3, 3, 1, 1, 1, 1, 1.0, A.ACT_RELU6, src, -1, ws, we, name=f"dw{idx}")

    chain = [pw(1, 0, 16, 48, A.ACT_RELU6, 0), pw(1, 1, 48, 24, A.ACT_NONE, 1),
             pw(1, 2, 24, 64, A.ACT_RELU6, 2), pw(1, 3, 64, 8, A.ACT_NONE, 3),
             pw(1, 4, 8, 40, A.ACT_HARDSWISH, 4), pw(1, 5, 40, 32, A.ACT_NONE, 5)]
    blocks = [pw(2, 0, 16, 64, A.ACT_RELU6, 0), dw(2, 1, 64, 1), pw(2, 2, 64, 24, A.ACT_NONE, 2),
              pw(2, 3, 24, 96, A.ACT_HARDSWISH, 3), dw(2, 4, 96, 4), pw(2, 5, 96, 32, A.ACT_NONE, 5),
              pw(2, 6, 32, 16, A.ACT_RELU, 6)]
    for name, layers, flag, launches in (("pairs", chain, npas.STACK_FUSE_POINTWISE, 3),
                                         ("blocks", blocks, npas.STACK_FUSE_INVERTED_RESIDUAL, 3)):
        N, HW, C = 5, 37, layers[0].C
        xs, xe = configs._tensor(31, 1, (N, HW, HW, C), 1.0, dtypes.BF16)
        w = configs.Workload("chained_" + name, dtypes.BF16, (N, HW, HW, C), xs, xe, layers)
        rounded, _ = oracle.run_stack(xe, layers, dtypes.BF16)
        fused, st = _run_stack_gpu(npas, torch, w, flag)
        plain, st0 = _run_stack_gpu(npas, torch, w, 0)
        assert st.num_launches() == launches and st0.num_launches() == len(layers)
        assert st.workspace_bytes(N) > 0
        n_f, e_f = helpers.check_stack_output(fused, rounded[-1], STACK_NORM_TOL)
        n_p, e_p = helpers.check_stack_output(plain, rounded[-1], STACK_NORM_TOL)
        print(f"  chained {name}: fused norm-wise {n_f:.3e} worst element {e_f:.3e}; unfused {n_p:.3e} / {e_p:.3e}", flush=True)
        again, _ = _run_stack_gpu(npas, torch, w, flag)
        np.testing.assert_array_equal(fused, again)


HS_CASES = [
    # hard-swish through every epilogue: name, N, H, W, C, F, KH, KW, stride, pad, Bf, Bc, rate, dtype, act, res, bias, variant, kernel
    (("hs_slab", 2, 11, 9, 24, 40, 3, 3, 1, 1, 8, 4, 2, dtypes.BF16, 3, True, True), None, "conv_slab_mfma"),
    (("hs_pointwise_ring", 3, 9, 11, 128, 136, 1, 1, 1, 0, 8, 4, 3, dtypes.BF16, 3, True, True), None, "pointwise_ring"),
    (("hs_spatial_ring", 3, 14, 14, 128, 64, 3, 3, 1, 1, 8, 4, 2, dtypes.BF16, 3, False, True), "spatial", "spatial_ring"),
    (("hs_resident_fp16", 2, 13, 11, 64, 40, 3, 3, 1, 1, 8, 4, 2, dtypes.F16, 3, True, False), "resident", "spatial_resident"),
    (("hs_smallm", 1, 7, 7, 128, 72, 3, 3, 1, 1, 8, 4, 3, dtypes.BF16, 3, True, True), None, "conv_smallm_mfma"),
    (("hs_smallc", 2, 21, 23, 3, 32, 5, 5, 2, 2, 8, 3, 2, dtypes.BF16, 3, False, True), None, "conv_smallc_mfma"),
    (("hs_gather", 1, 8, 8, 20, 18, 3, 3, 1, 1, 6, 4, 2, dtypes.BF16, 3, False, True), None, "conv_gather_mfma"),
    (("hs_fp32", 2, 9, 9, 8, 12, 3, 3, 1, 1, 4, 4, 2, dtypes.F32, 3, True, True), None, None),
    # the compiled epilogue variants of the spatial kernels (activation kind x residual), partial filter blocks, stride 2
    (("epi_spatial_hs_res", 3, 14, 14, 128, 128, 3, 3, 1, 1, 8, 4, 2, dtypes.BF16, 3, True, True), "spatial", "spatial_ring"),
    (("epi_spatial_s2_relu_res", 2, 28, 28, 64, 128, 3, 3, 2, 1, 8, 4, 2, dtypes.BF16, 1, True, True), "spatial", "spatial_ring"),
    (("epi_spatial_relu6_res_fp16_f200", 2, 9, 9, 64, 200, 3, 3, 1, 1, 8, 4, 3, dtypes.F16, 2, True, False), "spatial", "spatial_ring"),
    (("epi_resident_none_nores", 2, 12, 10, 64, 64, 3, 3, 1, 1, 8, 4, 2, dtypes.BF16, 0, False, True), "resident", "spatial_resident"),
    (("epi_pointwise_hs_nores_partial", 2, 7, 9, 64, 72, 1, 1, 1, 0, 8, 4, 2, dtypes.BF16, 3, False, False), None, None),
]


@pytest.mark.parametrize("case,variant,kernel", HS_CASES, ids=[c[0][0] for c in HS_CASES])
def test_hard_swish_epilogues(npas, torch, case, variant, kernel, force_variant):
    if variant:
        force_variant(variant)
    _run_edge_case(npas, torch, case, expect_kernel=kernel)


def test_full_size_config4_sampled_images(npas, torch):
    print("config4 full size, images 0/17/31", flush=True)
    w = configs.config4()
    L = w.layers[0]
    p = pack_layer(npas, L, w.dtype)
    helpers.check_metadata(oracle, L, p, w.dtype)
    y = from_dev(run_layer_gpu(npas, torch, L, p, to_dev(w.x_store, torch), w.x_shape, w.dtype), w.dtype)
    y = y.reshape(helpers.out_shape(L, w.x_shape))
    for n in (0, 17, 31):
        ref = oracle.round_to(oracle.conv2d_masked(w.x_exact[n:n + 1], L.w_exact, L.mask, 1, 1), w.dtype)
        err = rel_err(y[n:n + 1], ref)
        print(f"  image {n} err={err:.3e}", flush=True)
        assert err <= 1e-2


def test_config5_batch128_sampled_images(npas, torch):
    """The 50-layer stack's layers in the launch configuration the per-layer report times (batch 128: big tiles,
    both tile sizes of the streaming kernels, their stride-2 mode, the resident-weights kernel, the stem kernel), each on a seeded input of its real shape, checked
    on three of the 128 images (a layer's output for one image depends on that image only)."""
    w = configs.config5(batch=128)
    shapes = {0: w.x_shape}
    for i, L in enumerate(w.layers):
        shapes[i + 1] = helpers.out_shape(L, shapes[L.src])
    want = {"stem7x7": "conv_smallc_mfma", "s0b0_c3": "pointwise_ring", "s1b0_sc": "pointwise_ring", "s1b1_c2": "spatial_ring",
            "s2b1_c3": "pointwise_ring", "s2b0_c2": "spatial_ring", "s3b1_c1": "pointwise_ring", "s3b1_c2": "spatial_ring",
            "s0b1_c2": "spatial_resident"}
    seen = set()
    for i, L in enumerate(w.layers):
        if L.name not in want:
            continue
        seen.add(L.name)
        in_shape, oshape = shapes[L.src], shapes[i + 1]
        N, H, W, C = in_shape
        print(f"config5 batch 128 layer {i} {L.name} in={in_shape}", flush=True)
        xs, xe = dtypes.quantize(prng.normal(500 + i, 1, int(np.prod(in_shape))).reshape(in_shape), w.dtype)
        rs = re = None
        if L.res >= 0:
            rs, re = dtypes.quantize(prng.normal(500 + i, 2, int(np.prod(oshape))).reshape(oshape), w.dtype)
        p = pack_layer(npas, L, w.dtype)
        assert npas.conv2d_kernel_name(p, N, H, W, L.stride, L.pad) == want[L.name]
        y = run_layer_gpu(npas, torch, L, p, to_dev(xs, torch), in_shape, w.dtype, None if rs is None else to_dev(rs, torch))
        got = from_dev(y, w.dtype).reshape(oshape)
        for n in (0, 77, 127):
            ref = oracle.round_to(oracle.conv2d_masked(xe[n:n + 1], L.w_exact, L.mask, L.stride, L.pad, None,
                                                       None if re is None else re[n:n + 1], L.act), w.dtype)
            err = rel_err(got[n:n + 1], ref)
            print(f"  image {n} err={err:.3e}", flush=True)
            assert err <= TOL[w.dtype]
        del xs, xe, rs, re, y, got
        torch.cuda.empty_cache()
    assert seen == set(want)


def test_pools(npas, torch):
    # C = 24 takes the 8-channel vector path for 16-bit storage, C = 5 the scalar one
    for dtype, C in ((dtypes.BF16, 24), (dtypes.F16, 24), (dtypes.BF16, 5), (dtypes.F32, 24)):
        xs, xe = dtypes.quantize(prng.normal(9, 1, 2 * 9 * 11 * C).reshape(2, 9, 11, C), dtype)
        x = to_dev(xs, torch)
        y = new_dev((2, 5, 6, C), dtype, torch)
        npas.maxpool3x3s2(x, y, 2, 9, 11, C, dtype)
        np.testing.assert_array_equal(from_dev(y, dtype).reshape(2, 5, 6, C), oracle.maxpool3x3s2(xe))
        z = new_dev((2, C), dtype, torch)
        npas.global_avgpool(x, z, 2, 9, 11, C, dtype)
        assert rel_err(from_dev(z, dtype).reshape(2, C), oracle.round_to(oracle.global_avgpool(xe), dtype)) <= TOL[dtype]
