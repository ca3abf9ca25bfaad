"""Pins for the CPU oracle against things other than itself: a float64 library
convolution, an independently written im2col product, closed forms, and the
scheme invariants of paper sections 2.1 and 3.  The paper prints no worked
numeric example, so there are no golden tensors from it."""
import numpy as np
import pytest
import torch

import oracle
from workloads import dtypes, masks, prng


def rnd(seed, shape, sigma=1.0):
    return prng.normal(seed, 1, int(np.prod(shape)), sigma).reshape(shape)


def torch_conv(X, Wm, stride, pad, bias=None):
    x = torch.from_numpy(np.ascontiguousarray(X.transpose(0, 3, 1, 2)))
    y = torch.nn.functional.conv2d(x, torch.from_numpy(Wm), None if bias is None else torch.from_numpy(bias),
                                   stride=stride, padding=pad)
    return y.numpy().transpose(0, 2, 3, 1)


def im2col_conv(X, Wm, stride, pad):
    """Separately written check: explicit patch matrix times weight matrix."""
    N, H, W, C = X.shape
    F, _, KH, KW = Wm.shape
    Xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C))
    Xp[:, pad:pad + H, pad:pad + W] = X
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    cols = np.zeros((N, Ho, Wo, C, KH, KW))
    for y in range(Ho):
        for x in range(Wo):
            patch = Xp[:, y * stride:y * stride + KH, x * stride:x * stride + KW, :]   # N,KH,KW,C
            cols[:, y, x] = patch.transpose(0, 3, 1, 2)
    return cols.reshape(N * Ho * Wo, -1).dot(Wm.reshape(F, -1).T).reshape(N, Ho, Wo, F)


CASES = [
    # N, H, W, C, F, KH, KW, stride, pad, Bf, Bc, rate
    (2, 7, 9, 6, 8, 3, 3, 1, 1, 4, 4, 2),
    (1, 9, 8, 5, 7, 3, 3, 2, 1, 4, 2, 3),
    (2, 6, 5, 12, 10, 1, 1, 1, 0, 8, 4, 4),
    (1, 9, 7, 8, 6, 1, 1, 2, 0, 2, 8, 2),
    (1, 13, 15, 3, 8, 7, 7, 2, 3, 8, 4, 5),
    (1, 8, 10, 4, 4, 5, 3, 1, 2, 2, 2, 2.5),
    (1, 6, 6, 4, 4, 3, 3, 1, 0, 1, 1, 3),
]


@pytest.mark.parametrize("case", CASES)
def test_conv_matches_float64_library_convolution(case):
    N, H, W, C, F, KH, KW, s, p, Bf, Bc, rate = case
    X = rnd(11, (N, H, W, C))
    Wt = rnd(12, (F, C, KH, KW), 0.3)
    m = masks.block_punched_mask(F, C, KH, KW, Bf, Bc, rate, 77)
    bias = rnd(13, (F,))
    Y = oracle.conv2d_masked(X, Wt, m, s, p, bias)
    ref = torch_conv(X, Wt * m, s, p, bias)
    assert Y.shape == ref.shape
    np.testing.assert_allclose(Y, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("case", CASES[:5])
def test_conv_matches_im2col_product(case):
    N, H, W, C, F, KH, KW, s, p, Bf, Bc, rate = case
    X = rnd(21, (N, H, W, C))
    Wt = rnd(22, (F, C, KH, KW), 0.3)
    m = masks.block_punched_mask(F, C, KH, KW, Bf, Bc, rate, 78)
    Y = oracle.conv2d_masked(X, Wt, m, s, p)
    np.testing.assert_allclose(Y, im2col_conv(X, Wt * m, s, p), rtol=1e-12, atol=1e-12)


def test_all_ones_counts_surviving_inbounds_taps():
    F, C, Bf, Bc = 8, 8, 4, 4
    m = masks.block_punched_mask(F, C, 3, 3, Bf, Bc, 2, 5)
    X = np.ones((1, 6, 7, C))
    Y = oracle.conv2d_masked(X, np.ones((F, C, 3, 3)), m, 1, 1)
    for f in range(F):
        assert Y[0, 2, 3, f] == m[f].sum()                          # interior: K_eff of the group
        assert Y[0, 0, 0, f] == m[f][:, 1:, 1:].sum()               # top-left corner: taps kh,kw >= 1
        assert Y[0, 5, 6, f] == m[f][:, :2, :2].sum()               # bottom-right corner
        assert Y[0, 0, 3, f] == m[f][:, 1:, :].sum()                # top edge


def test_unit_impulse_reads_back_the_masked_kernel():
    F, C, KH, KW, p = 4, 3, 3, 5, 2
    Wt = rnd(31, (F, C, KH, KW))
    m = masks.block_punched_mask(F, C, KH, KW, 2, 3, 2, 6)
    y0, x0, c0 = 4, 5, 1
    X = np.zeros((1, 9, 11, C))
    X[0, y0, x0, c0] = 1.0
    Y = oracle.conv2d_masked(X, Wt, m, 1, p)
    Wm = Wt * m
    for y in range(Y.shape[1]):
        for x in range(Y.shape[2]):
            kh, kw = y0 - y + p, x0 - x + p
            exp = Wm[:, c0, kh, kw] if (0 <= kh < KH and 0 <= kw < KW) else np.zeros(F)
            np.testing.assert_array_equal(Y[0, y, x], exp)


def test_rate_one_is_dense_and_all_pruned_is_bias_only():
    X = rnd(41, (1, 5, 6, 4))
    Wt = rnd(42, (6, 4, 3, 3))
    bias = rnd(43, (6,))
    ones = masks.block_punched_mask(6, 4, 3, 3, 2, 2, 1, 3)
    assert ones.all()
    np.testing.assert_allclose(oracle.conv2d_masked(X, Wt, ones, 1, 1, bias), torch_conv(X, Wt, 1, 1, bias),
                               rtol=1e-12, atol=1e-12)
    Y = oracle.conv2d_masked(X, Wt, np.zeros_like(ones), 1, 1, bias)
    np.testing.assert_array_equal(Y, np.broadcast_to(bias, Y.shape))


def test_linearity_residual_and_activations():
    X1, X2 = rnd(51, (1, 5, 5, 4)), rnd(52, (1, 5, 5, 4))
    Wt = rnd(53, (4, 4, 3, 3))
    m = masks.block_punched_mask(4, 4, 3, 3, 2, 2, 2, 9)
    Y = oracle.conv2d_masked(2.0 * X1 - 3.0 * X2, Wt, m, 1, 1)
    np.testing.assert_allclose(Y, 2 * oracle.conv2d_masked(X1, Wt, m, 1, 1) - 3 * oracle.conv2d_masked(X2, Wt, m, 1, 1),
                               rtol=1e-12, atol=1e-12)
    R = rnd(54, Y.shape, 4.0)
    base = oracle.conv2d_masked(X1, Wt, m, 1, 1)
    np.testing.assert_allclose(oracle.conv2d_masked(X1, Wt, m, 1, 1, None, R, oracle.ACT_RELU),
                               np.maximum(base + R, 0.0), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.conv2d_masked(X1, Wt, m, 1, 1, None, R, oracle.ACT_RELU6),
                               np.clip(base + R, 0.0, 6.0), rtol=1e-13, atol=1e-13)
    assert (np.clip(base + R, 0, 6) == 6.0).any() and (np.clip(base + R, 0, 6) == 0.0).any()


def test_weights_under_the_mask_contribute_nothing():
    X = rnd(61, (1, 6, 6, 8))
    Wt = rnd(62, (8, 8, 3, 3))
    m = masks.block_punched_mask(8, 8, 3, 3, 4, 4, 3, 10)
    Wg = np.where(m == 1, Wt, np.nan)
    np.testing.assert_array_equal(oracle.conv2d_masked(X, Wg, m, 1, 1), oracle.conv2d_masked(X, Wt * m, m, 1, 1))
    mf = masks.fc_block_mask(10, 12, 4, 4, 2, 3)
    Wf = rnd(63, (10, 12))
    Xf = rnd(64, (3, 12))
    np.testing.assert_array_equal(oracle.fc_masked(Xf, np.where(mf == 1, Wf, np.inf), mf),
                                  oracle.fc_masked(Xf, Wf * mf, mf))


def test_fc_matches_matrix_product():
    Xf, Wf, b = rnd(71, (5, 70)), rnd(72, (37, 70)), rnd(73, (37,))
    mf = masks.fc_block_mask(37, 70, 16, 32, 5, 4)
    Y = oracle.fc_masked(Xf, Wf, mf, b, oracle.ACT_RELU)
    np.testing.assert_allclose(Y, np.maximum(Xf @ (Wf * mf).T + b, 0), rtol=1e-12, atol=1e-12)


def test_pattern_conv_equals_masked_conv_on_expanded_mask():
    F, C = 10, 12
    lib = masks.pattern_library(8, 5)
    assert (lib.sum(1) == 4).all() and (lib[:, 4] == 1).all() and len({tuple(r) for r in lib}) == 8
    m, ids = masks.pattern_mask(F, C, lib, 0.3, 6)
    Wt = rnd(81, (F, C, 3, 3))
    X = rnd(82, (2, 7, 6, C))
    rc, ids2 = oracle.validate_pattern(m, lib)
    assert rc == 0
    np.testing.assert_array_equal(ids, ids2)
    assert (ids == 255).sum() == 36
    w4 = oracle.pack_pattern(Wt, m)
    for s in (1, 2):
        Y1 = oracle.conv2d_pattern(X, w4, ids, lib, s, 1)
        Y2 = oracle.conv2d_masked(X, Wt, m, s, 1)
        np.testing.assert_allclose(Y1, Y2, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(Y1, torch_conv(X, Wt * m, s, 1), rtol=1e-12, atol=1e-12)
    # every kept kernel has exactly the pattern's entries, in ascending tap order
    for f in range(F):
        for c in range(C):
            if ids[f, c] == 255:
                assert not m[f, c].any() and not w4[f, c].any()
            else:
                taps = np.flatnonzero(lib[ids[f, c]])
                np.testing.assert_array_equal(w4[f, c], Wt[f, c].reshape(9)[taps])


def test_pools_match_library():
    X = rnd(91, (2, 9, 11, 5))
    xt = torch.from_numpy(np.ascontiguousarray(X.transpose(0, 3, 1, 2)))
    ref = torch.nn.functional.max_pool2d(xt, 3, 2, 1).numpy().transpose(0, 2, 3, 1)
    np.testing.assert_array_equal(oracle.maxpool3x3s2(X), ref)
    np.testing.assert_allclose(oracle.global_avgpool(X), X.mean(axis=(1, 2)), rtol=1e-13)
    Xneg = -np.abs(X) - 1.0          # padded cells must never win
    assert (oracle.maxpool3x3s2(Xneg) < 0).all()


@pytest.mark.parametrize("N,H,W,C,stride", [(2, 7, 9, 5, 1), (1, 8, 8, 16, 2), (2, 9, 6, 3, 2), (1, 1, 1, 4, 1), (1, 2, 5, 8, 1)])
def test_depthwise_matches_float64_grouped_library_convolution(N, H, W, C, stride):
    x = prng.normal(31, 1, N * H * W * C).reshape(N, H, W, C)
    w = prng.normal(31, 2, C * 9, 0.3).reshape(C, 3, 3)
    b = prng.normal(31, 3, C)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(w).reshape(C, 1, 3, 3),
                                     torch.from_numpy(b), stride=stride, padding=1, groups=C).permute(0, 2, 3, 1).numpy()
    got = oracle.dwconv3x3(x, w, stride, b)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_depthwise_closed_forms():
    C, H, W = 4, 5, 6
    w = prng.normal(32, 1, C * 9).reshape(C, 3, 3)
    # unit impulse in channel c0 at (y0, x0): the output is that channel's kernel, mirrored around the impulse,
    # and every other channel stays zero (channels do not mix)
    x = np.zeros((1, H, W, C))
    y0, x0, c0 = 2, 3, 1
    x[0, y0, x0, c0] = 1.0
    y = oracle.dwconv3x3(x, w)
    for oy in range(H):
        for ox in range(W):
            kh, kw = y0 - oy + 1, x0 - ox + 1
            want = w[c0, kh, kw] if 0 <= kh < 3 and 0 <= kw < 3 else 0.0
            assert y[0, oy, ox, c0] == want
    assert np.all(y[..., [0, 2, 3]] == 0.0)
    # all-ones input: interior = sum of the kernel, a corner = sum of the 2x2 taps that stay inside
    y = oracle.dwconv3x3(np.ones((1, H, W, C)), w)
    np.testing.assert_allclose(y[0, 2, 2], w.sum(axis=(1, 2)), rtol=1e-13)
    np.testing.assert_allclose(y[0, 0, 0], w[:, 1:, 1:].sum(axis=(1, 2)), rtol=1e-13)
    # it is the masked dense convolution whose weight tensor is diagonal in (filter, channel)
    xr = prng.normal(32, 2, 2 * H * W * C).reshape(2, H, W, C)
    dense = np.zeros((C, C, 3, 3))
    dense[np.arange(C), np.arange(C)] = w
    res = prng.normal(32, 3, 2 * 3 * 3 * C).reshape(2, 3, 3, C)
    a = oracle.dwconv3x3(xr, w, 2, None, res, oracle.ACT_RELU6)
    b = oracle.conv2d_masked(xr, dense, (dense != 0).astype(np.uint8), 2, 1, None, res, oracle.ACT_RELU6)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-13)


def test_rounding_matches_library_types_and_ties_to_even():
    v = np.concatenate([rnd(101, (20000,), 3.0), rnd(102, (2000,), 1e-39), rnd(103, (2000,), 1e30),
                        [1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -30, -1.0 - 2 ** -8, 0.0, 65520.0]])
    v32 = v.astype(np.float32).astype(np.float64)
    bf = torch.from_numpy(v32.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(oracle.round_to(v32, oracle.BF16), bf)
    np.testing.assert_array_equal(oracle.round_to(v32, oracle.BF16), dtypes.bf16_bits_to_f64(dtypes.f32_to_bf16_bits(v32)))
    small = v32[np.abs(v32) < 6e4]
    np.testing.assert_array_equal(oracle.round_to(small, oracle.F16), small.astype(np.float16).astype(np.float64))
    assert oracle.round_to([1.0 + 2 ** -8], 1)[0] == 1.0              # tie -> even (down)
    assert oracle.round_to([1.0 + 3 * 2 ** -8], 1)[0] == 1.0 + 2 ** -6  # tie -> even (up)
    assert oracle.round_to([65520.0], 2)[0] == np.inf
    np.testing.assert_array_equal(oracle.round_to(v, oracle.F32), v.astype(np.float32).astype(np.float64))


# ---------------------------------------------------------------- scheme definitions / packer

def unpack(grp, kpos, wc, F, C, KH, KW, Bf):
    Wd = np.zeros((F, C, KH, KW))
    for g in range(len(grp) - 1):
        for k in range(grp[g], grp[g + 1]):
            tap, c = divmod(int(kpos[k]), C)
            for j in range(Bf):
                if g * Bf + j < F:
                    Wd[g * Bf + j, c, tap // KW, tap % KW] = wc[k, j]
    return Wd


@pytest.mark.parametrize("F,C,KH,KW,Bf,Bc,rate", [(8, 8, 3, 3, 4, 4, 2), (10, 7, 3, 3, 4, 4, 3), (6, 16, 1, 1, 8, 8, 4),
                                                    (5, 3, 7, 7, 8, 4, 5), (4, 4, 3, 3, 1, 1, 2), (4, 4, 3, 3, 4, 4, 2)])
def test_pack_roundtrip_and_invariants(F, C, KH, KW, Bf, Bc, rate):
    m = masks.block_punched_mask(F, C, KH, KW, Bf, Bc, rate, 15)
    assert oracle.validate_block_punched(m, Bf, Bc) == 0
    Wt = rnd(111, (F, C, KH, KW))
    grp, kpos, wc = oracle.pack_block_punched(Wt, m, Bf)
    np.testing.assert_array_equal(unpack(grp, kpos, wc, F, C, KH, KW, Bf), Wt * m)
    G = -(-F // Bf)
    nnz = sum((grp[g + 1] - grp[g]) * (min(F, (g + 1) * Bf) - g * Bf) for g in range(G))
    assert nnz == m.sum()
    for g in range(G):                                   # ascending, unique positions per group
        assert (np.diff(kpos[grp[g]:grp[g + 1]]) > 0).all()
        np.testing.assert_array_equal(kpos[grp[g]:grp[g + 1]],
                                      np.flatnonzero(m[g * Bf].transpose(1, 2, 0).reshape(-1)))


def test_validators_reject_illegal_masks():
    m = masks.block_punched_mask(8, 8, 3, 3, 4, 4, 2, 16)
    bad = m.copy()
    f, c, kh, kw = 1, 2, 1, 1
    bad[f, c, kh, kw] ^= 1                                # one filter of a block disagrees
    assert oracle.validate_block_punched(bad, 4, 4) != 0
    assert oracle.validate_block_punched(m, 8, 4) != 0 or (m[:4] == m[4:]).all()   # wrong Bf is caught
    assert oracle.validate_block_punched(m, 2, 4) == 0    # finer filter groups stay legal
    bad = m.copy(); bad[0, 0, 0, 0] = 2
    assert oracle.validate_block_punched(bad, 4, 4) != 0
    mf = masks.fc_block_mask(32, 64, 16, 32, 4, 17)
    assert oracle.validate_fc_block(mf, 16, 32) == 0
    rows = mf.copy(); rows[3, :32] = 0                    # a pruned row inside a block is legal
    assert oracle.validate_fc_block(rows, 16, 32) == 0
    badf = mf.copy(); r, c = 5, int(np.flatnonzero(mf[5])[0]); badf[r, c] = 0   # a hole is not
    assert oracle.validate_fc_block(badf, 16, 32) != 0
    lib = masks.pattern_library(8, 5)
    mp, _ = masks.pattern_mask(6, 6, lib, 0.3, 18)
    assert oracle.validate_pattern(mp, lib)[0] == 0
    badp = mp.copy(); k = np.argwhere(mp.reshape(36, 9).sum(1) == 4)[0, 0]
    badp.reshape(36, 9)[k, 4] = 0                         # kernel loses its centre tap: 3 entries
    assert oracle.validate_pattern(badp, lib)[0] != 0


def test_generator_hits_the_requested_rates():
    m = masks.block_punched_mask(144, 24, 1, 1, 8, 8, 4, 1)
    assert m.sum() * 4 == m.size and (m.reshape(18, 8, 3, 8)[:, 0].sum(-1) == 2).all()
    mf = masks.fc_block_mask(1000, 1280, 16, 32, 5, 2)
    assert mf.sum() * 5 == mf.size
    per_block = mf[::16].reshape(63, 40, 32).sum(-1)
    assert set(np.unique(per_block)) == {6, 7}
    lib = masks.pattern_library(8, 3)
    mp, ids = masks.pattern_mask(128, 128, lib, 0.3, 4)
    assert (ids == 255).sum() == 4915 and mp.sum() == 4 * (128 * 128 - 4915)


def test_hard_swish_matches_its_formula():
    """hard-swish (paper section 5.1, Phase 1): v * clip(v + 3, 0, 6) / 6, here through every layer kind that
    takes an activation, with the residual added before it."""
    X = rnd(71, (1, 6, 5, 4), 2.0)
    Wt = rnd(72, (6, 4, 3, 3), 0.8)
    m = masks.block_punched_mask(6, 4, 3, 3, 2, 2, 2, 9)
    R = rnd(73, (1, 6, 5, 6), 3.0)
    base = oracle.conv2d_masked(X, Wt, m, 1, 1) + R
    hs = base * np.clip(base + 3.0, 0.0, 6.0) / 6.0
    np.testing.assert_allclose(oracle.conv2d_masked(X, Wt, m, 1, 1, None, R, oracle.ACT_HARDSWISH), hs, rtol=1e-13, atol=1e-13)
    assert (base < -3).any() and (base > 3).any() and ((base > -3) & (base < 3)).any()     # all three branches
    assert (hs[base <= -3] == 0).all() and np.allclose(hs[base >= 3], base[base >= 3], rtol=1e-15)
    Xf, Wf = rnd(74, (3, 12), 2.0), rnd(75, (10, 12))
    mf = masks.fc_block_mask(10, 12, 4, 4, 2, 3)
    v = Xf @ (Wf * mf).T
    np.testing.assert_allclose(oracle.fc_masked(Xf, Wf, mf, None, oracle.ACT_HARDSWISH), v * np.clip(v + 3, 0, 6) / 6,
                               rtol=1e-13, atol=1e-13)
    Wd = rnd(76, (4, 3, 3))
    d = oracle.dwconv3x3(X, Wd, 1)
    np.testing.assert_allclose(oracle.dwconv3x3(X, Wd, 1, None, None, oracle.ACT_HARDSWISH), d * np.clip(d + 3, 0, 6) / 6,
                               rtol=1e-13, atol=1e-13)


def _bf16(a):
    """float64 -> nearest bfloat16 (ties to even) -> float64, through PyTorch's cast (not the oracle's rounding)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def _assert_same_rounded(got, want, what=""):
    """Bit equality, except that a value the two float64 summation orders put on opposite sides of a rounding
    boundary may differ by one bfloat16 step (at most one element in a thousand; none for the seeds used here on
    the machine this was written on)."""
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, what
    bad = got != want
    if bad.any():
        assert bad.mean() <= 1e-3, f"{what}: {bad.sum()} of {bad.size} elements differ"
        assert (np.abs(got - want)[bad] <= np.abs(want)[bad] * 2.0 ** -7 + 1e-30).all(), what


def test_run_stack_wiring_and_rounding_against_plain_numpy():
    """The stack walker (which tensor a layer reads, which it adds, where activations are rounded) against the
    same networks written out by hand with NumPy matrix products, float64 library convolutions and PyTorch's
    bfloat16 cast.  The rounded tensors must agree bit for bit: a wrong src / res index, a residual added after
    the activation or a missed rounding between layers changes them."""
    from workloads import configs
    # (a) the 1x1 -> ReLU6 -> 1x1 pair: round_bf16(clip(x W1m^T, 0, 6)) W2m^T
    w = configs.config2(batch=1, HW=5)
    L1, L2 = w.layers
    rounded, raw = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    x = w.x_exact.reshape(-1, L1.C)
    W1m = (L1.w_exact * L1.mask).reshape(L1.F, L1.C)
    W2m = (L2.w_exact * L2.mask).reshape(L2.F, L2.C)
    mid = _bf16(np.clip(x @ W1m.T, 0.0, 6.0))
    out = mid @ W2m.T
    _assert_same_rounded(rounded[1].reshape(-1, L1.F), mid, "pair intermediate")
    np.testing.assert_allclose(raw[2].reshape(-1, L2.F), out, rtol=0, atol=1e-12)
    _assert_same_rounded(rounded[2].reshape(-1, L2.F), _bf16(out), "pair output")
    # (b) one bottleneck with a projection shortcut, the residual added before the ReLU, after a stem + max pool
    w = configs.config5(batch=1, HW=20, width=8, blocks=(1,), classes=10)
    names = [L.name for L in w.layers]
    assert names == ["stem7x7", "maxpool", "s0b0_c1", "s0b0_c2", "s0b0_sc", "s0b0_c3", "avgpool", "fc"]
    rounded, raw = oracle.run_stack(w.x_exact, w.layers, w.dtype)
    Ls = dict(zip(names, w.layers))

    def conv(x, L, res=None):
        y = torch_conv(x, L.w_exact * L.mask, L.stride, L.pad)
        if res is not None:
            y = y + res
        return _bf16(np.maximum(y, 0.0) if L.act == configs.ACT_RELU else y)

    t1 = conv(w.x_exact, Ls["stem7x7"])
    t2 = torch.nn.functional.max_pool2d(torch.from_numpy(t1.transpose(0, 3, 1, 2)), 3, 2, 1).numpy().transpose(0, 2, 3, 1)
    t3 = conv(t2, Ls["s0b0_c1"])
    t4 = conv(t3, Ls["s0b0_c2"])
    t5 = conv(t2, Ls["s0b0_sc"])                       # the shortcut reads the block input, no activation
    assert Ls["s0b0_sc"].act == configs.ACT_NONE and Ls["s0b0_c3"].res == 5 and Ls["s0b0_c3"].src == 4
    t6 = conv(t4, Ls["s0b0_c3"], res=t5)               # residual before the ReLU
    t7 = _bf16(t6.mean(axis=(1, 2)))
    Lf = Ls["fc"]
    t8 = t7 @ (Lf.w_exact * Lf.mask).reshape(Lf.F, Lf.C).T
    for i, t in enumerate((t1, t2, t3, t4, t5, t6, t7), start=1):
        _assert_same_rounded(rounded[i].reshape(t.shape), t, f"tensor {i} ({names[i - 1]})")
    np.testing.assert_allclose(raw[8], t8, rtol=0, atol=1e-12)
    _assert_same_rounded(rounded[8], _bf16(t8), "logits")
    assert np.abs(t6).max() > 0 and (t6 == 0).any()
    # (c) the cascade 1x1 -> depthwise 3x3 -> 1x1 with a bias per layer: the walker hands each layer its own bias,
    # which enters before the residual and the activation (a bias dropped, given to the wrong layer or added after
    # the clamp changes the rounded tensors)
    from workloads import sweeps
    for stride in (1, 2):
        w = sweeps.inverted_residual_block(batch=1, HW=7, stride=stride, bias=True)
        L1, L2, L3 = w.layers
        assert all(L.bias is not None and np.abs(L.bias).max() > 0.05 for L in w.layers)
        rounded, raw = oracle.run_stack(w.x_exact, w.layers, w.dtype)
        x = w.x_exact
        t1 = _bf16(np.clip(x.reshape(-1, L1.C) @ (L1.w_exact * L1.mask).reshape(L1.F, L1.C).T + L1.bias, 0.0, 6.0)).reshape(1, 7, 7, L1.F)
        dw = torch.nn.functional.conv2d(torch.from_numpy(t1.transpose(0, 3, 1, 2)), torch.from_numpy(L2.w_exact.reshape(L2.C, 1, 3, 3)),
                                        stride=stride, padding=1, groups=L2.C).numpy().transpose(0, 2, 3, 1)
        t2 = _bf16(np.clip(dw + L2.bias, 0.0, 6.0))
        t3 = t2.reshape(-1, L3.C) @ (L3.w_exact * L3.mask).reshape(L3.F, L3.C).T + L3.bias
        if stride == 1:
            t3 = t3 + x.reshape(-1, L1.C)
        _assert_same_rounded(rounded[1], t1, f"expansion, stride {stride}")
        _assert_same_rounded(rounded[2], t2, f"depthwise, stride {stride}")
        np.testing.assert_allclose(raw[3].reshape(t3.shape), t3, rtol=0, atol=1e-12)
