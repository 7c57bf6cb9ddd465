"""Helpers of the GPU parity tests: tolerances, tensor upload, sampled indices."""
import numpy as np
import torch

# spec tolerances: fp32 configs |gpu - ref| <= 1e-6 + 1e-5 |ref|; bf16-input config rtol 2e-2
TOL = {"f32": dict(rtol=1e-5, atol=1e-6), "bf16": dict(rtol=2e-2, atol=1e-3)}


def worst(gpu, ref, rtol, atol):
    """max over elements of |gpu-ref| / (atol + rtol |ref|); <= 1 passes."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    if gpu.size == 0:
        return 0.0
    assert np.isfinite(gpu).all(), "non-finite GPU output"
    return float((np.abs(gpu - ref) / (atol + rtol * np.abs(ref))).max())


def assert_close(gpu, ref, dtype="f32", what="", scale=1.0):
    t = TOL[dtype]
    w = worst(gpu, ref, t["rtol"] * scale, t["atol"] * scale)
    assert w <= 1.0, f"{what}: worst error is {w:.3g} x the tolerance (rtol={t['rtol']}, atol={t['atol']})"
    return w


def assert_dbias_close(got, ref, nterms, dtype="f32", what=""):
    """The bias gradient sums dl over all windows of a head (nterms of either sign).  Both sides get the same
    input bits, so the difference is rounding of the terms, which adds up like a random walk: relative 1e-5 of
    the largest entry plus c * sqrt(nterms), c = the rounding of one term (fp32 inputs: fp64 logits, ~1e-7 per
    term of magnitude <~ 1; bf16 inputs: fp32 logits of magnitude ~10, ~1e-6).  Returns the largest error."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    c = 2e-7 if dtype == "f32" else 2e-6
    tol = 1e-5 * np.abs(ref).max() + c * np.sqrt(nterms) + 1e-6
    err = float(np.abs(got - ref).max())
    assert err <= tol, f"{what}: dbias error {err:.3g} > {tol:.3g} (max |ref| {np.abs(ref).max():.3g}, {nterms} terms)"
    return err


# bf16-input cases: the inputs are the same bits on both sides and the kernels compute in fp32, so besides the
# stated bf16 tolerance (rtol 2e-2) the results must also agree at fp32 level: ten times the fp32 tolerance leaves
# room for fp32 logits of magnitude ~10 (1e-6 of rounding each), nothing more
BF16_FP32_LEVEL = 10.0


def assert_close_bf16_tight(gpu, ref, what="", scale=1.0):
    t = TOL["f32"]
    w = worst(gpu, ref, t["rtol"] * scale * BF16_FP32_LEVEL, t["atol"] * scale * BF16_FP32_LEVEL)
    assert w <= 1.0, f"{what}: {w * BF16_FP32_LEVEL:.3g} x the fp32 tolerance (bf16 inputs, fp32 arithmetic)"
    return w


def up(a, dtype="f32"):
    """numpy -> GPU tensor; bf16 inputs arrive as uint16 bit patterns."""
    if a is None:
        return None
    if dtype == "bf16" and a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def sample_windows(B, D, H, W, heads, n, seed=0, r=2):
    """n window indices (voxel*heads + head): all 8 corners, points on faces/edges, random interior."""
    rs = np.random.RandomState(seed)
    zs = np.concatenate([[0, D - 1, 0, D - 1], rs.randint(0, D, n)])
    ys = np.concatenate([[0, H - 1, H - 1, 0], rs.randint(0, H, n)])
    xs = np.concatenate([[0, W - 1, 0, W - 1], rs.randint(0, W, n)])
    # push a third of the random samples onto the border shell
    m = zs.size
    for arr, ext in ((zs, D), (ys, H), (xs, W)):
        sel = rs.rand(m) < 0.12
        arr[sel] = np.where(rs.rand(sel.sum()) < 0.5, rs.randint(0, min(r, ext), sel.sum()),
                            ext - 1 - rs.randint(0, min(r, ext), sel.sum()))
    bs = rs.randint(0, B, m)
    ss = rs.randint(0, heads, m)
    vox = ((bs * D + zs) * H + ys) * W + xs
    return np.unique(vox.astype(np.int64) * heads + ss)
