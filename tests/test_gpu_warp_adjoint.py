"""GPU parity of the warp adjoint (source and field gradients) against the CPU oracle, through the C ABI binding."""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_16526_amd import synth
from parity_util import assert_close, up

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def modet():
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2403_16526_amd import modet as m
    return m


@pytest.mark.parametrize("B,D,H,W,C,dtype,half", [
    (1, 6, 7, 9, 8, "f32", False), (2, 8, 10, 12, 8, "f32", True), (1, 5, 9, 33, 32, "f32", False),
    (1, 6, 8, 10, 3, "f32", False), (1, 6, 8, 10, 3, "f32", True), (1, 8, 6, 14, 16, "bf16", True),
    (1, 4, 5, 70, 16, "bf16", False), (1, 1, 1, 1, 4, "f32", False), (1, 2, 2, 2, 4, "f32", True),
    (1, 6, 7, 19, 6, "f32", False), (1, 6, 8, 18, 6, "bf16", True), (1, 5, 6, 11, 5, "f32", False),
    (1, 4, 6, 8, 250, "f32", True), (2, 5, 7, 9, 12, "bf16", False), (1, 4, 6, 8, 128, "f32", False),
    (1, 20, 18, 35, 2, "f32", False), (1, 18, 20, 34, 1, "f32", True), (2, 17, 33, 19, 8, "f32", False),
])
def test_warp_bwd_matches_oracle(modet, B, D, H, W, C, dtype, half):
    src = synth.normal(81, 0, (B, D, H, W, C))
    dout = synth.normal(82, 0, (B, D, H, W, C))
    fshape = (B, D // 2, H // 2, W // 2, 3) if half else (B, D, H, W, 3)
    field = (1.7 * synth.normal(83, 0, fshape)).astype(np.float32)
    field.reshape(-1)[::7] = np.round(field.reshape(-1)[::7])          # sample points exactly on voxels
    field.reshape(-1)[::11] *= 6.0                                      # some samples far outside
    if dtype == "bf16":
        src = synth.to_bf16_bits(src)
    ref_dsrc, ref_dfield = oracle.warp_bwd(src, field, dout, field_half_res=half, dtype=dtype)
    dsrc, dfield = modet.modet_warp_bwd(up(src, dtype), up(field), up(dout), field_half_res=half)
    only = modet.modet_warp_bwd(up(src, dtype), up(field), up(dout), field_half_res=half, want_dfield=False)
    tag = f"{(B, D, H, W, C)} {dtype} half={half}"
    assert_close(dsrc.cpu().numpy(), ref_dsrc, "f32", "dsrc " + tag)
    assert_close(only.cpu().numpy(), ref_dsrc, "f32", "dsrc alone " + tag)
    # the field gradient is a signed sum of 8 corners x C products (x up to 64 fine voxels per coarse entry):
    # its fp32 rounding is relative to the sum of the magnitudes, not to the result
    terms = 8.0 * np.sqrt(C) * (8.0 if half else 1.0)
    assert_close(dfield.cpu().numpy() / terms, ref_dfield / terms, "f32", "dfield " + tag)


@pytest.mark.parametrize("shift,half,std", [
    ((5.3, -7.6, 9.2), False, 1.2), ((-3.5, 4.5, -12.0), True, 1.0), ((40.0, 0.0, 0.0), False, 1.5),
    ((0.25, 0.5, -60.0), True, 0.5), ((-2.0, 3.0, 1.0), False, 4.0), ((0.0, 0.0, 0.0), True, 3.0),
])
def test_warp_bwd_large_coherent_displacement(modet, shift, half, std):
    """A smooth field around a large common shift (also one that points out of the volume, and rough ones): the
    source gradient's staged pass follows the local displacement, the atomic pass takes what strays from it."""
    B, D, H, W, C = 1, 36, 40, 50, 8
    src = synth.normal(91, 0, (B, D, H, W, C))
    dout = synth.normal(92, 0, (B, D, H, W, C))
    if half:
        field = synth.smooth_real_field(93, B, D // 2, H // 2, W // 2, std / 2) + np.float32(0.5) * np.asarray(shift, np.float32)
    else:
        field = synth.smooth_real_field(93, B, D, H, W, std) + np.asarray(shift, np.float32)
    field = np.ascontiguousarray(field, dtype=np.float32)
    ref_dsrc, ref_dfield = oracle.warp_bwd(src, field, dout, field_half_res=half)
    dsrc, dfield = modet.modet_warp_bwd(up(src), up(field), up(dout), field_half_res=half)
    only = modet.modet_warp_bwd(up(src), up(field), up(dout), field_half_res=half, want_dfield=False)
    assert_close(dsrc.cpu().numpy(), ref_dsrc, "f32", f"dsrc shift={shift}")
    assert_close(only.cpu().numpy(), ref_dsrc, "f32", f"dsrc alone shift={shift}")
    terms = 8.0 * np.sqrt(C) * (8.0 if half else 1.0)
    assert_close(dfield.cpu().numpy() / terms, ref_dfield / terms, "f32", f"dfield shift={shift}")


@pytest.mark.parametrize("rate,half", [(0.8, False), (0.95, False), (0.6, True), (1.0, False)])
def test_warp_bwd_contracting_field(modet, rate, half):
    """A field that pulls every voxel towards one point (rate 1: exactly onto it): many source voxels share
    their target voxels, so the staged pass has to apply entries of one column in turns."""
    B, D, H, W, C = 1, 20, 36, 40, 8
    src = synth.normal(94, 0, (B, D, H, W, C))
    dout = synth.normal(95, 0, (B, D, H, W, C))
    shape = (D // 2, H // 2, W // 2) if half else (D, H, W)
    grid = np.stack(np.meshgrid(*[np.arange(n, dtype=np.float64) for n in shape], indexing="ij"), axis=-1)
    centre = np.array([0.45 * n for n in shape])
    field = (-rate * (grid - centre) + 0.13)[None].astype(np.float32)      # (coarse voxels for the half-resolution case)
    field = np.ascontiguousarray(field)
    ref_dsrc, ref_dfield = oracle.warp_bwd(src, field, dout, field_half_res=half)
    dsrc, dfield = modet.modet_warp_bwd(up(src), up(field), up(dout), field_half_res=half)
    # up to a few thousand terms of either sign per element: compare relative to what was summed
    terms = np.sqrt(max(1.0, float(np.abs(ref_dsrc).max())))
    assert_close(dsrc.cpu().numpy() / terms, ref_dsrc / terms, "f32", f"dsrc rate={rate}", scale=4.0)
    t = 8.0 * np.sqrt(C) * (8.0 if half else 1.0)
    assert_close(dfield.cpu().numpy() / t, ref_dfield / t, "f32", f"dfield rate={rate}")


def test_warp_bwd_is_the_transpose_of_the_gpu_warp(modet):
    """<warp(x), y> = <x, warp_bwd(y)> with both sides computed on the GPU (fp32: 1e-5 of the magnitudes)."""
    B, D, H, W, C = 1, 12, 14, 40, 8
    x = up(synth.normal(84, 0, (B, D, H, W, C)))
    y = up(synth.normal(85, 0, (B, D, H, W, C)))
    field = up(synth.smooth_real_field(86, B, D, H, W, 2.0))
    lhs = (modet.modet_warp(x, field).double() * y.double()).sum().item()
    rhs = (x.double() * modet.modet_warp_bwd(x, field, y, want_dfield=False).double()).sum().item()
    assert abs(lhs - rhs) <= 1e-5 * (x.abs().double() * y.abs().double()).sum().item() ** 0.5 * 10


def test_warp_bwd_full_volume(modet):
    """config-3 shape (160x192x224, C=8), half-resolution field as the pyramid uses it: every element."""
    c = synth.make_config(3)
    B, D, H, W, C = c["B"], c["D"], c["H"], c["W"], c["C"]
    coarse = synth.smooth_real_field(12, B, D // 2, H // 2, W // 2, 1.0)
    dout = c["Q"]                                  # any N(0,1) tensor of the right shape
    dsrc, dfield = modet.modet_warp_bwd(up(c["K"]), up(coarse), up(dout), field_half_res=True)
    ref_dsrc, ref_dfield = oracle.warp_bwd(c["K"], coarse, dout, field_half_res=True)
    assert_close(dsrc.cpu().numpy(), ref_dsrc, "f32", "dsrc")
    terms = 8.0 * np.sqrt(C) * 8.0
    assert_close(dfield.cpu().numpy() / terms, ref_dfield / terms, "f32", "dfield")
