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
