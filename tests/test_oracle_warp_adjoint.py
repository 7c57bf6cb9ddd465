"""Pins of the oracle's warp adjoint (the step before the operator in the pyramid of Section 3.1, differentiated)
against the oracle's own, already pinned, forward warp: the transpose identity for the source gradient and
finite differences for the field gradient, which are exact here because the warp is linear in each displacement
component as long as the sample point stays inside its cell."""
import numpy as np
import pytest

import oracle
from paper_2403_16526_amd import synth


def case(B, D, H, W, C, half, seed=0):
    src = synth.normal(71 + seed, 0, (B, D, H, W, C), dtype=np.float64)
    y = synth.normal(72 + seed, 0, (B, D, H, W, C), dtype=np.float64)
    fshape = (B, D // 2, H // 2, W // 2, 3) if half else (B, D, H, W, 3)
    field = (1.3 * synth.normal(73 + seed, 0, fshape)).astype(np.float32)
    return src, y, field


@pytest.mark.parametrize("half", [False, True])
@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_source_gradient_is_the_transpose_of_the_warp(half, dtype):
    """<warp(x), y> = <x, warp^T(y)> for every x: checked with a second random x, which a mere copy of the
    forward loop with the roles swapped would also pass only if weights and indices are the same."""
    src, y, field = case(2, 6, 8, 10, 5, half)
    if dtype == "f32":
        src = src.astype(np.float32)
    x2 = synth.normal(74, 0, src.shape, dtype=np.float64).astype(src.dtype)
    dsrc = oracle.warp_bwd(src, field, y, field_half_res=half, dtype=dtype, want_dfield=False)
    for x in (src, x2):
        lhs = float((oracle.warp(x, field, field_half_res=half, dtype=dtype) * y).sum())
        rhs = float((x.astype(np.float64) * dsrc).sum())
        assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    # samples that leave the volume read zeros and hand nothing back: the total weight is below the voxel count
    ones = oracle.warp_bwd(src, field, np.ones_like(y), field_half_res=half, dtype=dtype, want_dfield=False)
    assert 0.3 * src.size < ones.sum() < src.size


def test_field_gradient_matches_exact_central_differences():
    """Displacements are put on odd multiples of 1/512, so +-1/1024 never crosses a voxel boundary: the central
    difference of the (piecewise linear) loss is then its derivative up to fp64 rounding."""
    B, D, H, W, C = 1, 5, 6, 7, 3
    src, y, field = case(B, D, H, W, C, False, seed=3)
    field = (np.round(field * 256.0) / 256.0 + 1.0 / 512.0).astype(np.float32)
    _, dfield = oracle.warp_bwd(src, field, y, dtype="f64")
    eps = np.float32(1.0 / 1024.0)
    rng = np.random.default_rng(5)
    for idx in rng.choice(field.size, 60, replace=False):
        fp, fm = field.copy(), field.copy()
        fp.reshape(-1)[idx] += eps
        fm.reshape(-1)[idx] -= eps
        lp = (oracle.warp(src, fp, dtype="f64") * y).sum()
        lm = (oracle.warp(src, fm, dtype="f64") * y).sum()
        assert abs((lp - lm) / (2.0 * float(eps)) - dfield.reshape(-1)[idx]) <= 1e-9


def test_half_resolution_field_gradient():
    """(i) finite differences on coarse entries (a coarse entry moves up to 4x4x4 fine voxels, each linearly while
    it stays in its cell; with a step of 2^-14 a boundary crossing is rare and costs O(step));
    (ii) the chain rule: the same gradient through the oracle's 2x upsampling -- fine-grid field gradient at the
    upsampled displacement, pulled back with the transpose of upsample2x (built column by column)."""
    B, D, H, W, C = 1, 6, 8, 6, 4
    src, y, coarse = case(B, D, H, W, C, True, seed=6)
    _, dcoarse = oracle.warp_bwd(src, coarse, y, field_half_res=True, dtype="f64")
    eps = np.float32(2.0 ** -14)
    scale = np.abs(dcoarse).max()
    bad = 0
    for idx in range(0, coarse.size, 3):
        fp, fm = coarse.copy(), coarse.copy()
        fp.reshape(-1)[idx] += eps
        fm.reshape(-1)[idx] -= eps
        lp = (oracle.warp(src, fp, field_half_res=True, dtype="f64") * y).sum()
        lm = (oracle.warp(src, fm, field_half_res=True, dtype="f64") * y).sum()
        fd = (lp - lm) / (float(fp.reshape(-1)[idx]) - float(fm.reshape(-1)[idx]))
        if abs(fd - dcoarse.reshape(-1)[idx]) > 1e-6 * scale:
            bad += 1
    assert bad <= 1
    # (ii) upsample2x is linear: column j of its matrix is upsample2x(e_j)
    fine = oracle.upsample2x(coarse)
    _, dfine = oracle.warp_bwd(src, fine.astype(np.float32), y, dtype="f64")
    pulled = np.empty(coarse.size)
    for j in range(coarse.size):
        e = np.zeros(coarse.size, np.float32)
        e[j] = 1.0
        pulled[j] = (oracle.upsample2x(e.reshape(coarse.shape)) * dfine).sum()
    # the full-resolution call rounds the upsampled field to fp32 (1e-7 relative on the displacements)
    np.testing.assert_allclose(pulled.reshape(coarse.shape), dcoarse, rtol=0, atol=2e-5 * scale)


def test_zero_gradient_where_nothing_is_read():
    """a displacement that throws every sample out of the volume: no source voxel receives anything, and the field
    gradient is zero as well (all eight corners are padding)."""
    src, y, field = case(1, 4, 4, 4, 2, False)
    field[...] = 50.0
    dsrc, dfield = oracle.warp_bwd(src, field, y, dtype="f64")
    assert not dsrc.any() and not dfield.any()
