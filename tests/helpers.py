"""Shared plumbing of the GPU parity tests: device buffers via PyTorch, calls
through the C-ABI binding, and the error metric."""
import numpy as np

from workloads import dtypes
from workloads.harness import (bias_tensors, from_dev, new_dev, out_shape, pack_layer, run_layer_gpu,  # noqa: F401
                               stack_descs, to_dev)

TOL = {dtypes.F32: 1e-5, dtypes.BF16: 1e-2, dtypes.F16: 2e-3}


def rel_err(gpu, ref):
    """max_i |g_i - o_i| / max(|o_i|, tau), tau = 1e-3 * max_j |o_j| (element-wise
    relative error with a floor so that cancelled sums do not divide by ~0)."""
    gpu, ref = np.asarray(gpu, np.float64), np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    tau = 1e-3 * max(np.abs(ref).max(), 1e-30)
    assert np.isfinite(gpu).all(), "non-finite GPU output"
    return float((np.abs(gpu - ref) / np.maximum(np.abs(ref), tau)).max())


def check_metadata(oracle, L, packed, dtype):
    """Bit-exact comparison of the library's canonical compact form with the oracle's."""
    e = packed.export()
    Bf = 1 if L.scheme == "pattern" else min(L.Bf, L.F)
    grp, kpos, wc = oracle.pack_block_punched(L.w_exact, L.mask, Bf)
    np.testing.assert_array_equal(e["grp_ptr"], grp)
    np.testing.assert_array_equal(e["k_pos"], kpos)
    got = dtypes.storage_to_f64(e["w_compact"], dtype)
    np.testing.assert_array_equal(got.view(np.int64), wc.view(np.int64))
    if L.scheme == "pattern":
        rc, ids = oracle.validate_pattern(L.mask, L.library)
        assert rc == 0
        np.testing.assert_array_equal(e["pat_id"], ids)
        w4 = oracle.pack_pattern(L.w_exact, L.mask)
        np.testing.assert_array_equal(dtypes.storage_to_f64(e["w4"], dtype).view(np.int64), w4.view(np.int64))


def bf16_step(v):
    """Spacing of bfloat16 values at |v| (8 significand bits; the smallest normal's spacing below it)."""
    a = np.maximum(np.abs(np.asarray(v, np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def check_two_layer_pointwise(got, ref, mid_rounded, W2m, tol=1e-2, flips=2):
    """Element-wise check of a fused 1x1 -> act -> 1x1 launch whose intermediate never leaves the kernel.
    The kernel's fp32 sum and the oracle's fp64 sum of an intermediate value can land on opposite sides of a
    rounding boundary; the intermediate then differs by one bfloat16 step s(mid), and an output that reads it
    moves by |W2[f, c]| s(mid[p, c]).  Such flips are rare (the two sums differ by ~1e-7 relative, the boundaries
    are 2^-8 apart), so an output is allowed `flips` of them, the largest ones, on top of the per-layer tolerance:
        |g - o| <= tol max(|o|, tau) + sum of the `flips` largest |W2[f, c]| s(mid[p, c]) over c.
    Returns (plain relative error, share of elements beyond the plain tolerance)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    F2 = W2m.shape[0]
    g, o, mid = got.reshape(-1, F2), ref.reshape(-1, F2), np.asarray(mid_rounded, np.float64).reshape(-1, W2m.shape[1])
    assert np.isfinite(g).all(), "non-finite GPU output"
    tau = 1e-3 * max(np.abs(o).max(), 1e-30)
    base = tol * np.maximum(np.abs(o), tau)
    step = bf16_step(mid)                                           # [pixels][C2]
    allow = np.zeros_like(o)
    for f in range(F2):
        terms = step * np.abs(W2m[f])[None, :]
        allow[:, f] = np.sort(np.partition(terms, -flips, axis=1)[:, -flips:], axis=1).sum(axis=1)
    diff = np.abs(g - o)
    worst = float((diff / np.maximum(np.abs(o), tau)).max())
    beyond = float((diff > base).mean())
    bad = diff > base + allow
    assert not bad.any(), f"{bad.sum()} outputs differ by more than the tolerance plus {flips} intermediate rounding flips (worst plain error {worst:.3e})"
    assert beyond <= 1e-3, f"{beyond:.2e} of the outputs are beyond the plain tolerance: more than rounding flips explain"
    norm = float(diff.max() / np.abs(o).max())
    assert norm <= tol, f"norm-wise error {norm:.3e}"
    return worst, beyond


def check_stack_output(got, ref, tol=1e-2, quantile=0.999):
    """A stack end to end: norm-wise error within tol, all but 1 - quantile of the elements within tol element-wise
    (an intermediate value rounded the other way moves a few outputs by more; see check_two_layer_pointwise).
    Returns (norm-wise error, worst element-wise error)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape and np.isfinite(got).all()
    tau = 1e-3 * max(np.abs(ref).max(), 1e-30)
    rel = np.abs(got - ref) / np.maximum(np.abs(ref), tau)
    norm = float(np.abs(got - ref).max() / np.abs(ref).max())
    assert norm <= tol, f"norm-wise error {norm:.3e}"
    q = float(np.quantile(rel, quantile))
    assert q <= tol, f"{quantile} quantile of the element-wise error is {q:.3e}"
    return norm, float(rel.max())
