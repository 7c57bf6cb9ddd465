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
    (1, 4, 6, 8, 250, "f32", True), (2, 5, 7, 9, 12, "bf16", False),
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
