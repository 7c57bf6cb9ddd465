"""Pins of the oracle's displacement-field composition (Section 3.1) and of its scaling-and-squaring integration
(Section 3.3.2, Eq. 6) against closed forms: cases where trilinear interpolation is exact (integer shifts,
affine fields) and flows whose solution is known (constant and linear velocity)."""
import numpy as np

import oracle
from paper_2403_16526_amd import synth


def grid(D, H, W):
    z, y, x = np.meshgrid(np.arange(D), np.arange(H), np.arange(W), indexing="ij")
    return np.stack([z, y, x], axis=-1).astype(np.float64)[None]          # [1,D,H,W,3]


def test_zero_inner_field_returns_the_outer_field():
    outer = synth.smooth_real_field(3, 2, 6, 7, 9, 1.5)
    out = oracle.compose(outer, np.zeros_like(outer))
    np.testing.assert_array_equal(out, outer.astype(np.float64))


def test_integer_shift_reads_the_outer_field_at_the_shifted_voxel():
    """inner = constant integer vector o: out[p] = o + outer[p + o] where p + o is inside, o elsewhere (zero padding);
    a transposed axis or a flipped sign moves the slice."""
    outer = synth.smooth_real_field(4, 1, 7, 8, 9, 2.0).astype(np.float64)
    o = (1, -2, 3)
    inner = np.broadcast_to(np.array(o, np.float32), outer.shape).copy()
    out = oracle.compose(outer, inner)
    want = np.broadcast_to(np.array(o, np.float64), outer.shape).copy()
    want[:, :-1, 2:, :-3] += outer[:, 1:, :-2, 3:]
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-15)


def test_affine_outer_field_is_reproduced_exactly():
    """Trilinear interpolation reproduces a function that is linear in the coordinates, so with outer(x) = A x + c:
    out[p] = inner[p] + A (p + inner[p]) + c wherever all eight corners are inside.  A is not symmetric: swapped
    axes, swapped weights or a wrong component order all change the result."""
    D, H, W = 12, 13, 14
    A = np.array([[0.02, -0.01, 0.03], [0.015, 0.01, -0.02], [-0.03, 0.025, 0.005]])
    c = np.array([0.3, -0.2, 0.1])
    g = grid(D, H, W)
    outer = (g @ A.T + c).astype(np.float32)
    inner = synth.smooth_real_field(5, 1, D, H, W, 0.8)
    out = oracle.compose(outer, inner)
    q = g + inner.astype(np.float64)
    want = inner.astype(np.float64) + outer_exact(outer, q, A, c)
    m = np.all((q >= 0) & (q <= np.array([D - 1, H - 1, W - 1])), axis=-1)
    assert m.mean() > 0.7
    # outer itself was rounded to fp32 (~1e-8 on values < 1): the interpolant of the rounded samples
    np.testing.assert_allclose(out[m], want[m], rtol=0, atol=2e-7)


def outer_exact(outer, q, A, c):
    return q @ A.T + c


def test_constant_velocity_integrates_to_itself():
    """d(phi)/dt = v with v constant: phi(1) = v.  Each squaring step doubles the field exactly.  The zero padding
    outside the volume enters at the faces and moves inwards by the interpolation footprint (one voxel) plus the
    displacement per step, so only voxels more than T + 2 from every face are compared."""
    v = np.broadcast_to(np.array([0.5, -0.25, 0.75], np.float32), (1, 24, 25, 26, 3)).copy()
    for T in (0, 1, 4, 7):
        phi = oracle.integrate_velocity(v, T)
        m = T + 2
        np.testing.assert_allclose(phi[:, m:-m, m:-m, m:-m], v[:, m:-m, m:-m, m:-m], rtol=0, atol=1e-6)


def test_linear_velocity_integrates_to_the_compound_interest_formula():
    """v_z = c (z - z0), other components zero.  One Euler step of size 1/2^T is x -> (1 + c/2^T)(x - z0) + z0 and
    every squaring squares the factor (interpolation is exact on linear fields), so
    phi_T(z) = ((1 + c/2^T)^(2^T) - 1)(z - z0), which tends to (e^c - 1)(z - z0), the solution of Eq. 6."""
    D, H, W, c, z0 = 48, 5, 6, 0.2, 24
    z = np.arange(D, dtype=np.float64)
    v = np.zeros((1, D, H, W, 3), np.float32)
    v[..., 0] = (c * (z - z0)).astype(np.float32)[None, :, None, None]
    sl = slice(8, D - 8)                      # paths that stay inside: |phi| < 0.23 * 16 = 3.6 there
    for T in (1, 3, 7, 10):
        phi = oracle.integrate_velocity(v, T)
        want = ((1.0 + c / 2 ** T) ** (2 ** T) - 1.0) * (z - z0)
        np.testing.assert_allclose(phi[0, sl, 2, 3, 0], want[sl], rtol=2e-6, atol=2e-6)
        assert np.abs(phi[..., 1:]).max() == 0.0
    # (1 + c/n)^n = e^c (1 - c^2 / 2n + ...): 1.1e-4 relative on e^c - 1 at n = 2^10
    np.testing.assert_allclose(phi[0, sl, 2, 3, 0], (np.exp(c) - 1.0) * (z - z0)[sl], rtol=1.5e-4, atol=1e-6)


def test_flow_of_the_negated_velocity_is_the_inverse():
    """exp(v) o exp(-v) = identity for the exact flow.  Scaling and squaring approaches it as the step 1/2^T
    shrinks, down to the error of resampling the field on the grid (a few percent of a voxel for this field of
    up to two voxels): no squaring at all (T = 0, phi = v) is ten times worse."""
    D, H, W, m = 40, 42, 44, 8
    v = synth.smooth_real_field(6, 1, D, H, W, 0.5)
    res = {}
    for T in (0, 2, 7):
        fwd = oracle.integrate_velocity(v, T)
        bwd = oracle.integrate_velocity(-v, T)
        r = oracle.compose(fwd.astype(np.float32), bwd.astype(np.float32))
        res[T] = np.abs(r[:, m:-m, m:-m, m:-m]).max()
    assert res[0] > 0.3 and res[2] < 0.5 * res[0] and res[7] < 0.1 * res[0] and res[7] < 0.05
