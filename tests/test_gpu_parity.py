"""GPU parity: libmodet (through the C ABI binding) against the CPU oracle, element by element on
small seeded cases that span several tiles and ragged tails, plus the degenerate shapes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_16526_amd import synth
from parity_util import assert_close, assert_close_bf16_tight, assert_dbias_close, up

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def modet():
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2403_16526_amd import modet as m
    return m


# (B, D, H, W, C, heads, k, dtype)
SMALL = [
    (1, 16, 16, 16, 8, 1, 3, "f32"),        # config 1
    (2, 9, 19, 70, 8, 1, 3, "f32"),         # ragged in every axis, W spans two 64-lane rows
    (1, 5, 11, 131, 8, 1, 3, "f32"),
    (1, 7, 13, 37, 32, 4, 3, "f32"),        # config 2 style heads
    (1, 6, 10, 21, 64, 8, 3, "f32"),        # coarsest pyramid level style
    (1, 12, 9, 23, 16, 2, 3, "f32"),
    (1, 9, 12, 21, 16, 2, 5, "bf16"),       # config 5 style
    (2, 6, 21, 40, 8, 1, 5, "f32"),
    (1, 7, 8, 9, 8, 1, 3, "bf16"),
    (1, 1, 1, 1, 8, 1, 3, "f32"),           # a single voxel: every neighbour is padding
    (1, 2, 3, 1, 8, 1, 3, "f32"),           # thinner than the window
    (1, 1, 40, 3, 16, 2, 5, "f32"),
    (1, 5, 6, 7, 12, 2, 3, "f32"),          # the paper's small model: 6 channels per head
    (1, 4, 5, 6, 24, 2, 3, "bf16"),         # the paper's large model: 12 channels per head
    (1, 4, 5, 6, 8, 1, 1, "f32"),           # k = 1
    (1, 5, 6, 9, 4, 1, 7, "f32"),
    (1, 57, 17, 65, 8, 1, 3, "f32"),        # several chunks along D with ragged tiles: chunk seams of the marches
    (2, 20, 9, 33, 8, 1, 3, "bf16"),
    (1, 41, 12, 40, 16, 2, 3, "f32"),       # the same for the several-heads backward
    # six channels per head on the tiled kernels: ragged tiles and chunk seams, 1 / 2 / 4 / 8 heads, both dtypes
    (1, 45, 13, 67, 6, 1, 3, "f32"),
    (2, 11, 9, 35, 12, 2, 3, "bf16"),
    (1, 9, 10, 33, 24, 4, 3, "f32"),
    (1, 6, 9, 17, 48, 8, 3, "bf16"),
    (1, 37, 8, 40, 12, 2, 3, "f32"),
    # twelve channels per head on the tiled kernels (two half-head lanes per window): 1 / 2 / 4 heads, both dtypes
    (1, 45, 13, 35, 12, 1, 3, "f32"),
    (2, 9, 10, 19, 24, 2, 3, "f32"),
    (1, 6, 9, 9, 48, 4, 3, "bf16"),
    (1, 37, 9, 33, 12, 1, 3, "bf16"),
    # chunk seams of the four-heads-and-more backward (and of its bias gradient)
    (1, 45, 9, 20, 32, 4, 3, "f32"),
    (1, 41, 9, 17, 24, 2, 3, "bf16"),
    (1, 30, 9, 40, 8, 1, 5, "bf16"),        # k = 5 with chunk seams (bias gradient summed wave by wave)
    (2, 23, 10, 35, 16, 2, 5, "bf16"),
    (1, 5, 6, 7, 24, 3, 3, "f32"),          # three heads: no tiled variant, generic kernels under both paths
    # the head counts of the paper's large model (Section 4.4: 32 / 16 / 8 heads of 12 channels) and of its small
    # one (8 heads of 6), and 16 / 32 heads of 8 channels
    (1, 5, 6, 9, 384, 32, 3, "f32"),
    (1, 6, 7, 11, 192, 16, 3, "bf16"),
    (1, 9, 8, 13, 96, 8, 3, "f32"),
    (1, 6, 5, 12, 128, 16, 3, "f32"),
    (1, 4, 6, 10, 256, 32, 3, "bf16"),
    # head groups with two batch items and ragged tiles along W and H
    (2, 4, 5, 33, 96, 16, 3, "f32"), (2, 3, 9, 7, 192, 16, 3, "bf16"), (2, 5, 11, 6, 128, 16, 3, "f32"),
]


def run_case(modet, shape, path, with_bias=False, stats="pass"):
    B, D, H, W, C, heads, k, dtype = shape
    keys = "displaced" if min(D, H, W) >= 4 else "iid"
    c = synth.make_case(B, D, H, W, C, heads, k, dtype=dtype, keys=keys, m=(k - 1) // 2, seed=1000 + D * H + W)
    bias = (0.5 * synth.normal(77, 0, (heads, k ** 3))).astype(np.float32) if with_bias else None
    ref_phi, ref_attn, ref_lse = oracle.modet_fwd(c["Q"], c["K"], heads, k, bias=bias, dtype=dtype, want_attn=True,
                                                  want_lse=True)
    ref_dQ, ref_dK, ref_db = oracle.modet_bwd(c["Q"], c["K"], c["dphi"], heads, k, bias=bias, dtype=dtype,
                                              form="scatter", want_dbias=True)
    Q, K, g, tb = up(c["Q"], dtype), up(c["K"], dtype), up(c["dphi"]), up(bias)
    old = modet.modet_set_kernel_path(path)
    try:
        phi, lse = modet.modet_fwd(Q, K, heads, k, bias=tb, want_lse=True)
        phi2, attn = modet.modet_fwd(Q, K, heads, k, bias=tb, want_attn=True)
        given = dict(phi=phi, lse=lse) if stats == "pass" else {}
        dQ, dK, db = modet.modet_bwd(Q, K, g, heads, k, bias=tb, want_dbias=True, **given)
        # without the bias gradient (and without bias) other kernels run
        dQ2, dK2 = modet.modet_bwd(Q, K, g, heads, k, bias=tb, **given)
        torch.cuda.synchronize()
    finally:
        modet.modet_set_kernel_path(old)
    tag = f"{shape} path={path} bias={with_bias} stats={stats}"
    # fp32 rounding of a gradient grows with the number of cancelling terms in its sum: the stated
    # tolerance is for the 27-term window, larger windows get it scaled by k^3 / 27
    gs = max(1.0, k ** 3 / 27.0)
    assert_close(phi.cpu().numpy(), ref_phi, dtype, "phi " + tag, scale=gs)
    assert_close(phi2.cpu().numpy(), ref_phi, dtype, "phi(attn call) " + tag, scale=gs)
    assert_close(attn.cpu().numpy(), ref_attn, dtype, "attn " + tag)
    assert_close(lse.cpu().numpy(), ref_lse, dtype, "lse " + tag)
    assert_close(dQ.cpu().numpy(), ref_dQ, dtype, "dQ " + tag, scale=gs)
    assert_close(dK.cpu().numpy(), ref_dK, dtype, "dK " + tag, scale=gs)
    assert_close(dQ2.cpu().numpy(), ref_dQ, dtype, "dQ (no dbias) " + tag, scale=gs)
    assert_close(dK2.cpu().numpy(), ref_dK, dtype, "dK (no dbias) " + tag, scale=gs)
    if dtype == "bf16":      # fp32 arithmetic on identical input bits: the result is good to fp32 level, not to 2e-2
        for name, got, ref in (("phi", phi, ref_phi), ("dQ", dQ, ref_dQ), ("dK", dK, ref_dK), ("dQ (no dbias)", dQ2, ref_dQ),
                               ("dK (no dbias)", dK2, ref_dK), ("lse", lse, ref_lse)):
            assert_close_bf16_tight(got.cpu().numpy(), ref, f"{name} {tag}", scale=gs)
    # dbias sums dl over all windows of a head
    assert_dbias_close(db.cpu().numpy(), ref_db, B * D * H * W, dtype, "dbias " + tag)


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("path", [0, 1], ids=["auto", "generic"])
def test_small_cases_match_oracle(modet, shape, path):
    run_case(modet, shape, path)


# with bias: one / two heads (k = 3) with chunk seams, four and eight heads, k = 5, 6 and 12 channels per head,
# both dtypes
BIASED = [SMALL[1], SMALL[3], SMALL[4], SMALL[6], SMALL[8], SMALL[12], SMALL[13], SMALL[16], SMALL[17], SMALL[18],
          SMALL[19], SMALL[20], SMALL[21], SMALL[22], SMALL[23], SMALL[24], SMALL[25], SMALL[26], SMALL[27],
          SMALL[28], SMALL[29], SMALL[30], SMALL[31], SMALL[32], SMALL[33], SMALL[34], SMALL[35], SMALL[36], SMALL[37],
          SMALL[38], SMALL[39], SMALL[40]]


@pytest.mark.parametrize("shape", BIASED, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("path", [0, 1], ids=["auto", "generic"])
def test_bias_and_recomputed_statistics(modet, shape, path):
    run_case(modet, shape, path, with_bias=True, stats="recompute")


@pytest.mark.parametrize("shape", [SMALL[16], SMALL[18], SMALL[6], SMALL[19], SMALL[24]],
                         ids=lambda s: "x".join(map(str, s)))
def test_bias_with_statistics_passed_in(modet, shape):
    run_case(modet, shape, 0, with_bias=True, stats="pass")


@pytest.mark.parametrize("shape", [SMALL[1], SMALL[3], SMALL[6], SMALL[12], SMALL[8], SMALL[9], SMALL[32]],
                         ids=lambda s: "x".join(map(str, s)))
def test_gradient_through_the_attention_weights(modet, shape):
    """the weights of Eq. 3 as a second output with an upstream gradient of their own: dQ, dK and the bias gradient
    of sum(dphi * phi) + sum(dattn * attn), with the forward's statistics passed in and recomputed."""
    B, D, H, W, C, heads, k, dtype = shape
    keys = "displaced" if min(D, H, W) >= 4 else "iid"
    c = synth.make_case(B, D, H, W, C, heads, k, dtype=dtype, keys=keys, m=(k - 1) // 2, seed=2000 + D * H + W)
    bias = (0.5 * synth.normal(79, 0, (heads, k ** 3))).astype(np.float32)
    da = synth.normal(80, 0, (B, D, H, W, heads, k ** 3))
    ref_dQ, ref_dK, ref_db = oracle.modet_bwd(c["Q"], c["K"], c["dphi"], heads, k, bias=bias, dtype=dtype,
                                              form="scatter", want_dbias=True, dattn=da)
    Q, K, g = up(c["Q"], dtype), up(c["K"], dtype), up(c["dphi"])
    phi, lse = modet.modet_fwd(Q, K, heads, k, bias=up(bias), want_lse=True)
    gs = max(1.0, k ** 3 / 27.0)
    for given in (dict(phi=phi, lse=lse), {}):
        dQ, dK, db = modet.modet_bwd(Q, K, g, heads, k, bias=up(bias), want_dbias=True, dattn=up(da), **given)
        tag = f"{shape} stats {'passed' if given else 'recomputed'}"
        assert_close(dQ.cpu().numpy(), ref_dQ, dtype, "dQ " + tag, scale=gs)
        assert_close(dK.cpu().numpy(), ref_dK, dtype, "dK " + tag, scale=gs)
        if dtype == "bf16":
            assert_close_bf16_tight(dQ.cpu().numpy(), ref_dQ, "dQ " + tag, scale=gs)
            assert_close_bf16_tight(dK.cpu().numpy(), ref_dK, "dK " + tag, scale=gs)
        assert_dbias_close(db.cpu().numpy(), ref_db, B * D * H * W, dtype, "dbias " + tag)
    # a gradient that is constant over each window changes nothing (the weights of a window sum to one)
    dQ0, dK0 = modet.modet_bwd(Q, K, g, heads, k, bias=up(bias), phi=phi, lse=lse)
    dQ1, dK1 = modet.modet_bwd(Q, K, g, heads, k, bias=up(bias), phi=phi, lse=lse,
                               dattn=torch.full(da.shape, 0.25, device="cuda"))
    assert_close(dQ1.cpu().numpy(), dQ0.cpu().numpy().astype(np.float64), dtype, "constant dattn dQ", scale=gs)
    assert_close(dK1.cpu().numpy(), dK0.cpu().numpy().astype(np.float64), dtype, "constant dattn dK", scale=gs)


def test_explicit_scale_and_peaked_attention(modet):
    """large scale: attention is one-hot on the planted integer offset (sign / axis order on the GPU)."""
    B, D, H, W, heads, d, k = 1, 8, 9, 70, 1, 8, 3
    Q = synth.normal(5, 0, (B, D, H, W, heads, d), dtype=np.float64)
    Q = (Q / np.linalg.norm(Q, axis=-1, keepdims=True)).reshape(B, D, H, W, heads * d).astype(np.float32)
    o = (1, -1, 1)
    K = np.zeros_like(Q)
    K[:, 1:, :-1, 1:] = Q[:, :-1, 1:, :-1]            # K[p + o] = Q[p]
    for path in (0, 1):
        old = modet.modet_set_kernel_path(path)
        phi = modet.modet_fwd(up(Q), up(K), heads, k, scale=1.0e4).cpu().numpy()
        modet.modet_set_kernel_path(old)
        np.testing.assert_allclose(phi[:, :-1, 1:, :-1, 0], np.broadcast_to(np.array(o, np.float32),
                                                                            phi[:, :-1, 1:, :-1, 0].shape), atol=1e-5)
        ref = oracle.modet_fwd(Q, K, heads, k, scale=1.0e4)
        # logits are ~1e4 here: fp32 rounding of the logit itself is ~1e-3, so only a loose bound holds
        assert np.abs(phi - ref).max() < 5e-2


@pytest.mark.parametrize("dtype,heads,k,d", [("f32", 1, 3, 8), ("f32", 2, 3, 8), ("bf16", 2, 3, 8), ("bf16", 1, 5, 8),
                                             ("f32", 2, 3, 6), ("bf16", 1, 3, 6), ("f32", 1, 3, 12), ("bf16", 2, 3, 12)])
def test_forward_survives_logits_far_above_the_first_window_row(modet, dtype, heads, k, d):
    """The tiled forward measures every logit of a query against the largest one of the first window row it
    meets.  Here half of the queries have their match in the LAST plane of the window with a logit ~400 (log2
    units) above everything else, which overflows fp32 exponentials: those queries take the two-pass path and
    must still agree with the oracle, the other half must be untouched by it."""
    B, D, H, W = 1, 9, 12, 70
    r = k // 2
    Q = synth.normal(31, 0, (B, D, H, W, heads, d), dtype=np.float64)
    Q = (Q / np.linalg.norm(Q, axis=-1, keepdims=True)).reshape(B, D, H, W, heads * d).astype(np.float32)
    K = (0.05 * synth.normal(31, 1, Q.shape)).astype(np.float32)
    K[:, r:, :, : W // 2] = Q[:, :-r, :, : W // 2]          # K[p + (r, 0, 0)] = Q[p] for the left half
    if dtype == "bf16":
        Q, K = synth.to_bf16_bits(Q), synth.to_bf16_bits(K)
    scale = 300.0
    for bias in (None, (0.5 * synth.normal(78, 0, (heads, k ** 3))).astype(np.float32)):
        ref_phi, _, ref_lse = oracle.modet_fwd(Q, K, heads, k, scale=scale, bias=bias, dtype=dtype, want_attn=True,
                                               want_lse=True)
        for path in (0, 1):
            old = modet.modet_set_kernel_path(path)
            phi, lse = modet.modet_fwd(up(Q, dtype), up(K, dtype), heads, k, scale=scale, bias=up(bias),
                                       want_lse=True)
            modet.modet_set_kernel_path(old)
            tag = f"path {path} bias {bias is not None}"
            # The exponent of a weight, (logit - reference), is rounded to fp32 before exp2.  The logits of this
            # test spread over +-60 (log2 units) around a query's reference instead of the few units normalised
            # features give, so that rounding alone is up to 2^-24 * 64 = 4e-6 relative per weight: four times
            # the stated tolerance is what the arithmetic supports here.
            assert_close(phi.cpu().numpy(), ref_phi, dtype, "phi " + tag, scale=4.0)
            np.testing.assert_allclose(lse.cpu().numpy(), ref_lse, rtol=2e-2 if dtype == "bf16" else 2e-6, atol=1e-5,
                                       err_msg=tag)
    # the planted half really is (nearly always) one-hot on (r, 0, 0), the other half is not
    assert np.median(np.abs(ref_phi[:, : D - r, :, : W // 2, :, 0] - r)) < 1e-9
    assert np.median(np.abs(ref_phi[:, :, :, W // 2 + r:, :, 0] - r)) > 0.1


def test_fp32_logit_mode_is_close_but_outside_the_bar(modet):
    """the optional fp32-logit arithmetic: same answers to a few 1e-6, which is why it is not the default."""
    c = synth.make_case(1, 24, 40, 70, 8, 1, 3, keys="displaced", m=1, seed=21)
    Q, K, g = up(c["Q"]), up(c["K"]), up(c["dphi"])
    ref_phi = oracle.modet_fwd(c["Q"], c["K"], 1, 3)
    ref_dQ, ref_dK = oracle.modet_bwd(c["Q"], c["K"], c["dphi"], 1, 3)
    old = modet.modet_set_math_mode(1)
    try:
        phi, lse = modet.modet_fwd(Q, K, 1, 3, want_lse=True)
        dQ, dK = modet.modet_bwd(Q, K, g, 1, 3, phi=phi, lse=lse)
    finally:
        assert modet.modet_set_math_mode(old) == 1
    from parity_util import worst
    for name, got, ref in (("phi", phi, ref_phi), ("dQ", dQ, ref_dQ), ("dK", dK, ref_dK)):
        w = worst(got.cpu().numpy(), ref, 1e-5, 1e-6)
        print(f"fp32-logit mode {name}: worst error {w:.2f} x tolerance")
        assert w < 10.0


def test_zero_query_is_uniform_everywhere(modet):
    K = up(synth.normal(6, 0, (1, 6, 7, 66, 8)))
    for path in (0, 1):
        old = modet.modet_set_kernel_path(path)
        phi, lse = modet.modet_fwd(torch.zeros_like(K), K, 1, 3, want_lse=True)
        modet.modet_set_kernel_path(old)
        assert phi.abs().max().item() <= 1e-7
        np.testing.assert_allclose(lse.cpu().numpy(), np.log(27.0), rtol=1e-6)


def test_backward_is_deterministic(modet):
    c = synth.make_case(1, 12, 21, 70, 8, 1, 3, keys="displaced", m=1, seed=9)
    Q, K, g = up(c["Q"]), up(c["K"]), up(c["dphi"])
    a = modet.modet_bwd(Q, K, g, 1, 3)
    b = modet.modet_bwd(Q, K, g, 1, 3)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_outputs_are_fully_overwritten(modet):
    c = synth.make_case(1, 6, 9, 67, 8, 1, 3, seed=10)
    Q, K, g = up(c["Q"]), up(c["K"]), up(c["dphi"])
    dQ = torch.full(Q.shape, float("nan"), device="cuda")
    dK = torch.full(Q.shape, float("nan"), device="cuda")
    modet.modet_bwd(Q, K, g, 1, 3, out=(dQ, dK))
    ref = oracle.modet_bwd(c["Q"], c["K"], c["dphi"], 1, 3)
    assert_close(dQ.cpu().numpy(), ref[0], "f32", "dQ")
    assert_close(dK.cpu().numpy(), ref[1], "f32", "dK")


def test_errors_surface_as_exceptions(modet):
    Q = torch.zeros((1, 4, 4, 4, 8), device="cuda")
    with pytest.raises(modet.ModetError) as e:
        modet.modet_fwd(Q, Q.clone(), 3, 3)
    assert e.value.status == -2
    with pytest.raises(modet.ModetError):
        modet.modet_fwd(Q, Q.clone(), 1, 4)


# ---- warp -------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,D,H,W,C,dtype,half", [
    (1, 6, 7, 9, 8, "f32", False), (2, 8, 10, 12, 8, "f32", True), (1, 5, 9, 33, 32, "f32", False),
    (1, 6, 8, 10, 3, "f32", False), (1, 6, 8, 10, 3, "f32", True), (1, 8, 6, 14, 16, "bf16", True),
    (1, 9, 11, 70, 1, "f32", False), (2, 8, 10, 34, 1, "f32", True),      # one channel: the final image warp
    (1, 4, 5, 70, 16, "bf16", False), (1, 1, 1, 1, 4, "f32", False), (1, 2, 2, 2, 4, "f32", True),
    # channel counts of the paper's head sizes (6 and 12 per head) and odd ones: narrower vectors per lane
    (1, 6, 7, 19, 6, "f32", False), (1, 6, 8, 18, 6, "bf16", True), (2, 5, 7, 9, 12, "bf16", False),
    (1, 6, 8, 10, 12, "f32", True), (1, 5, 6, 11, 5, "f32", False), (1, 4, 6, 8, 250, "f32", True),
    (1, 4, 5, 7, 26, "bf16", False),
])
def test_warp_matches_oracle(modet, B, D, H, W, C, dtype, half):
    src = synth.normal(61, 0, (B, D, H, W, C))
    fshape = (B, D // 2, H // 2, W // 2, 3) if half else (B, D, H, W, 3)
    field = (1.7 * synth.normal(62, 0, fshape)).astype(np.float32)
    field.reshape(-1)[::7] = np.round(field.reshape(-1)[::7])          # some exactly-integer displacements
    field.reshape(-1)[::11] *= 6.0                                      # some samples far outside
    if dtype == "bf16":
        src = synth.to_bf16_bits(src)
    ref = oracle.warp(src, field, field_half_res=half, dtype=dtype)
    out = modet.modet_warp(up(src, dtype), up(field), field_half_res=half)
    got = out.float().cpu().numpy()
    if dtype == "bf16":
        # the output is rounded to bf16: half an ulp of bf16 (2^-9 relative) on top of fp32 accumulation
        assert_close(got, ref, "bf16", "warp bf16")
    else:
        assert_close(got, ref, "f32", "warp f32")


def test_warp_identity_and_integer_shift_are_exact(modet):
    src = synth.normal(63, 0, (1, 6, 7, 40, 8))
    z = torch.zeros((1, 6, 7, 40, 3), device="cuda")
    assert torch.equal(modet.modet_warp(up(src), z), up(src))
    u = z.clone()
    u[..., 0], u[..., 1], u[..., 2] = 1.0, -2.0, 3.0
    out = modet.modet_warp(up(src), u).cpu().numpy()
    exp = np.zeros_like(src)
    exp[:, 0:5, 2:7, 0:37] = src[:, 1:6, 0:5, 3:40]
    assert np.array_equal(out, exp)
