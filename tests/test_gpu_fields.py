"""GPU parity of the displacement-field composition (Section 3.1) and of the scaling-and-squaring integration
(Section 3.3.2, Eq. 6) against the CPU oracle, through the C ABI binding."""
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


SHAPES = [(1, 16, 16, 16), (2, 9, 19, 70), (1, 5, 11, 131), (1, 1, 1, 1), (1, 2, 3, 1), (1, 33, 20, 65)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_compose_matches_oracle(modet, shape):
    B, D, H, W = shape
    outer = synth.smooth_real_field(21, B, D, H, W, 2.0)
    inner = synth.smooth_real_field(22, B, D, H, W, 1.5)       # some samples leave the volume: zero padding
    out = modet.modet_compose(up(outer), up(inner))
    assert_close(out.cpu().numpy(), oracle.compose(outer, inner), "f32", f"compose {shape}")
    t = up(inner)
    out = modet.modet_compose(t, t)                              # a field with itself, from one buffer
    assert_close(out.cpu().numpy(), oracle.compose(inner, inner), "f32", f"self-compose {shape}")


@pytest.mark.parametrize("shape", [(1, 16, 16, 16), (2, 10, 18, 70), (1, 6, 12, 130), (1, 2, 2, 2), (1, 2, 4, 2),
                                   (1, 34, 20, 66)], ids=lambda s: "x".join(map(str, s)))
def test_compose_with_half_resolution_outer_field(modet, shape):
    """the coarser level's field as the outer field: upsampled 2x inside the kernel (odd / ragged coarse extents,
    samples that leave the volume, a volume of one coarse voxel)."""
    B, D, H, W = shape
    coarse = synth.smooth_real_field(27, B, D // 2, H // 2, W // 2, 1.5)
    inner = synth.smooth_real_field(28, B, D, H, W, 1.7)
    out = modet.modet_compose(up(coarse), up(inner), outer_half_res=True)
    assert_close(out.cpu().numpy(), oracle.compose(coarse, inner, outer_half_res=True), "f32", f"compose-up {shape}")


@pytest.mark.parametrize("T", [0, 1, 2, 5, 7])
@pytest.mark.parametrize("shape", [(1, 16, 16, 16), (2, 9, 19, 70), (1, 2, 3, 1)], ids=lambda s: "x".join(map(str, s)))
def test_integrate_velocity_matches_oracle(modet, shape, T):
    B, D, H, W = shape
    v = synth.smooth_real_field(23, B, D, H, W, 1.5)
    phi = modet.modet_integrate_velocity(up(v), T)
    # both sides round every intermediate field to fp32; a difference of one step is doubled by the next along
    # with the field itself, so the error relative to the field grows by about one step's worth per step
    assert_close(phi.cpu().numpy(), oracle.integrate_velocity(v, T), "f32", f"integrate {shape} T={T}",
                 scale=max(1, T))


def test_integrate_velocity_with_caller_buffers(modet):
    """out and tmp given by the caller; the result must land in out for odd and even T."""
    B, D, H, W = 1, 12, 13, 14
    v = up(synth.smooth_real_field(24, B, D, H, W, 1.0))
    for T in (2, 3):
        out, tmp = torch.full_like(v, 7.0), torch.full_like(v, 9.0)
        got = modet.modet_integrate_velocity(v, T, out=out, tmp=tmp)
        assert got.data_ptr() == out.data_ptr()
        assert_close(out.cpu().numpy(), oracle.integrate_velocity(v.cpu().numpy(), T), "f32", f"T={T}", scale=T)


def test_compose_and_integrate_full_volume(modet):
    """the config-3 volume (160x192x224): every element."""
    B, D, H, W = 1, 160, 192, 224
    outer = synth.smooth_real_field(25, B, D, H, W, 2.0)
    inner = synth.smooth_real_field(26, B, D, H, W, 1.5)
    out = modet.modet_compose(up(outer), up(inner))
    assert_close(out.cpu().numpy(), oracle.compose(outer, inner), "f32", "compose")
    phi = modet.modet_integrate_velocity(up(inner), 7)
    assert_close(phi.cpu().numpy(), oracle.integrate_velocity(inner, 7), "f32", "integrate T=7", scale=7)
    coarse = synth.smooth_real_field(29, B, D // 2, H // 2, W // 2, 1.0)
    out = modet.modet_compose(up(coarse), up(inner), outer_half_res=True)
    assert_close(out.cpu().numpy(), oracle.compose(coarse, inner, outer_half_res=True), "f32", "compose-up")
