"""GPU parity on the benchmark configurations at their full sizes, in the launch configuration
bench.py times (automatic kernel path, statistics handed from the forward to the backward)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_16526_amd import synth
from parity_util import assert_close, assert_close_bf16_tight, assert_dbias_close, sample_windows, up

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


@pytest.fixture(scope="module")
def modet():
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2403_16526_amd import modet as m
    return m


def gpu_fwd_bwd(modet, c):
    dtype, heads, k = c["dtype"], c["heads"], c["k"]
    Q, K, g = up(c["Q"], dtype), up(c["K"], dtype), up(c["dphi"])
    phi, lse = modet.modet_fwd(Q, K, heads, k, want_lse=True)
    dQ, dK = modet.modet_bwd(Q, K, g, heads, k, phi=phi, lse=lse)
    torch.cuda.synchronize()
    return phi, lse, dQ, dK


@pytest.mark.parametrize("no", [1, 2, 3])
def test_fp32_configs_full_volume(modet, no):
    """configs 1-3: every element of phi, lse, dQ, dK against the oracle."""
    c = synth.make_config(no)
    heads, k = c["heads"], c["k"]
    phi, lse, dQ, dK = gpu_fwd_bwd(modet, c)
    ref_phi, ref_lse = oracle.modet_fwd(c["Q"], c["K"], heads, k, want_lse=True)
    assert_close(phi.cpu().numpy(), ref_phi, "f32", f"config {no} phi")
    assert_close(lse.cpu().numpy(), ref_lse, "f32", f"config {no} lse")
    del ref_phi, ref_lse
    ref_dQ, ref_dK = oracle.modet_bwd(c["Q"], c["K"], c["dphi"], heads, k, form="gather")
    assert_close(dQ.cpu().numpy(), ref_dQ, "f32", f"config {no} dQ")
    assert_close(dK.cpu().numpy(), ref_dK, "f32", f"config {no} dK")


def test_config3_with_bias_and_bias_gradient_full_volume(modet):
    """config 3 with a bias B (Eq. 3) of the size a trained one would have: every element of phi, lse, dQ, dK,
    and the bias gradient, a sum over all 6.9 million voxels whose terms largely cancel."""
    c = synth.make_config(3)
    heads, k = c["heads"], c["k"]
    bias = (0.5 * synth.normal(79, 0, (heads, k ** 3))).astype(np.float32)
    Q, K, g, tb = up(c["Q"]), up(c["K"]), up(c["dphi"]), up(bias)
    phi, lse = modet.modet_fwd(Q, K, heads, k, bias=tb, want_lse=True)
    dQ, dK, db = modet.modet_bwd(Q, K, g, heads, k, bias=tb, phi=phi, lse=lse, want_dbias=True)
    torch.cuda.synchronize()
    ref_phi, ref_lse = oracle.modet_fwd(c["Q"], c["K"], heads, k, bias=bias, want_lse=True)
    assert_close(phi.cpu().numpy(), ref_phi, "f32", "phi")
    assert_close(lse.cpu().numpy(), ref_lse, "f32", "lse")
    del ref_phi, ref_lse
    ref_dQ, ref_dK, ref_db = oracle.modet_bwd(c["Q"], c["K"], c["dphi"], heads, k, bias=bias, form="scatter",
                                              want_dbias=True)
    assert_close(dQ.cpu().numpy(), ref_dQ, "f32", "dQ")
    assert_close(dK.cpu().numpy(), ref_dK, "f32", "dK")
    # each entry sums ~7e6 terms of either sign and magnitude up to ~1: the fp32 terms themselves carry ~1e-7
    # relative rounding each, so the sum is good to ~1e-7 * sqrt(7e6) * rms(term) in absolute terms
    err = np.abs(db.cpu().numpy() - ref_db)
    print("dbias: max |ref|", np.abs(ref_db).max(), "max abs err", err.max())
    assert err.max() <= 1e-5 * np.abs(ref_db).max() + 2e-4


def test_config3_without_forward_statistics(modet):
    """the backward alone (statistics recomputed into the workspace) on a slab of config 3."""
    c = synth.make_config(3, D=24)
    Q, K, g = up(c["Q"]), up(c["K"]), up(c["dphi"])
    dQ, dK = modet.modet_bwd(Q, K, g, 1, 3)
    ref_dQ, ref_dK = oracle.modet_bwd(c["Q"], c["K"], c["dphi"], 1, 3, form="gather")
    assert_close(dQ.cpu().numpy(), ref_dQ, "f32", "dQ")
    assert_close(dK.cpu().numpy(), ref_dK, "f32", "dK")


def test_config5_bf16_k5_sampled(modet):
    """config 5 (2x192x160x192, C=16, 2 heads, k=5, bf16 inputs): sampled windows, corners and faces included."""
    c = synth.make_config(5)
    B, D, H, W, C, heads, k = (c[n] for n in ("B", "D", "H", "W", "C", "heads", "k"))
    phi, lse, dQ, dK = gpu_fwd_bwd(modet, c)
    idx = sample_windows(B, D, H, W, heads, 6000, seed=5, r=2)
    ref_phi, ref_lse = oracle.modet_fwd_at(c["Q"], c["K"], idx, heads, k, dtype="bf16")
    ref_dQ, ref_dK = oracle.modet_bwd_at(c["Q"], c["K"], c["dphi"], idx, heads, k, dtype="bf16")
    d = C // heads
    t = torch.from_numpy(idx).cuda()
    got_phi = phi.reshape(-1, 3)[t].cpu().numpy()
    got_lse = lse.reshape(-1)[t].cpu().numpy()
    got_dQ = dQ.reshape(-1, d)[t].cpu().numpy()
    got_dK = dK.reshape(-1, d)[t].cpu().numpy()
    assert_close(got_phi, ref_phi, "bf16", "config 5 phi")
    assert_close(got_lse, ref_lse, "bf16", "config 5 lse")
    assert_close(got_dQ, ref_dQ, "bf16", "config 5 dQ")
    assert_close(got_dK, ref_dK, "bf16", "config 5 dK")
    # the inputs are bit-identical on both sides, so the error is in fact at fp32 level: report it
    w = max(np.abs(got_phi - ref_phi).max(), np.abs(got_dQ - ref_dQ).max(), np.abs(got_dK - ref_dK).max())
    print(f"config 5 max abs error over {idx.size} sampled windows: {w:.3g}")
    assert w < 1e-4
    # properties that hold at any size
    assert torch.isfinite(phi).all() and torch.isfinite(dQ).all() and torch.isfinite(dK).all()
    assert phi.abs().max().item() <= 2.0 + 1e-5


def test_config5_full_slabs_at_both_faces(modet):
    """config 5, batch item 1: every element of the 12 planes at each D face of the full-size run.  The oracle
    runs on the 16-plane sub-volume those outputs depend on: k = 5 reaches two planes, and dK of a key reaches
    four (the queries two planes away, whose softmax spans two more)."""
    c = synth.make_config(5)
    B, D, H, W, C, heads, k = (c[n] for n in ("B", "D", "H", "W", "C", "heads", "k"))
    phi, lse, dQ, dK = gpu_fwd_bwd(modet, c)
    n, halo = 12, 4
    for lo, hi, keep in ((0, n + halo, slice(0, n)), (D - n - halo, D, slice(halo, n + halo))):
        Qs, Ks, gs = (c[name][1:2, lo:hi].copy() for name in ("Q", "K", "dphi"))
        ref_phi, ref_lse = oracle.modet_fwd(Qs, Ks, heads, k, dtype="bf16", want_lse=True)
        ref_dQ, ref_dK = oracle.modet_bwd(Qs, Ks, gs, heads, k, dtype="bf16", form="gather")
        for name, got, ref in (("phi", phi, ref_phi), ("lse", lse, ref_lse), ("dQ", dQ, ref_dQ), ("dK", dK, ref_dK)):
            g_ = got[1:2, lo:hi][:, keep].cpu().numpy()
            r_ = ref[:, keep]
            assert_close(g_, r_, "bf16", f"config 5 slab {lo}:{hi} {name}")
            assert_close_bf16_tight(g_, r_, f"config 5 slab {lo}:{hi} {name}", scale=k ** 3 / 27.0)


def test_config5_shape_bias_gradient(modet):
    """the k = 5 bias gradient (summed wave by wave inside the dQ march) at config 5's in-plane extents: a
    24-plane volume of the same batch, H, W, channels and heads, with a bias, every entry against the oracle."""
    c = synth.make_config(5, D=24)
    B, D, H, W, C, heads, k = (c[n] for n in ("B", "D", "H", "W", "C", "heads", "k"))
    bias = (0.5 * synth.normal(synth.BASE_SEED + 5, 9, (heads, k ** 3))).astype(np.float32)
    Q, K, g = up(c["Q"], "bf16"), up(c["K"], "bf16"), up(c["dphi"])
    phi, lse = modet.modet_fwd(Q, K, heads, k, bias=up(bias), want_lse=True)
    dQ, dK, db = modet.modet_bwd(Q, K, g, heads, k, bias=up(bias), phi=phi, lse=lse, want_dbias=True)
    ref_dQ, ref_dK, ref_db = oracle.modet_bwd(c["Q"], c["K"], c["dphi"], heads, k, bias=bias, dtype="bf16",
                                              form="scatter", want_dbias=True)
    assert_close_bf16_tight(dQ.cpu().numpy(), ref_dQ, "dQ", scale=k ** 3 / 27.0)
    assert_close_bf16_tight(dK.cpu().numpy(), ref_dK, "dK", scale=k ** 3 / 27.0)
    err = assert_dbias_close(db.cpu().numpy(), ref_db, B * D * H * W, "bf16", "config-5 shape")
    print(f"k=5 dbias: max |ref| {np.abs(ref_db).max():.4g}, max abs error {err:.3g}")


def test_warp_config3_shape_full_volume(modet):
    c = synth.make_config(3)
    B, D, H, W = c["B"], c["D"], c["H"], c["W"]
    field = synth.smooth_real_field(11, B, D, H, W, 1.5)
    out = modet.modet_warp(up(c["K"]), up(field))
    assert_close(out.cpu().numpy(), oracle.warp(c["K"], field), "f32", "warp full res field")
    coarse = synth.smooth_real_field(12, B, D // 2, H // 2, W // 2, 1.0)
    out = modet.modet_warp(up(c["K"]), up(coarse), field_half_res=True)
    assert_close(out.cpu().numpy(), oracle.warp(c["K"], coarse, field_half_res=True), "f32", "warp half res field")


def _check_level_calls(store, levels, it):
    """every operator call of every level, re-run by the oracle on the GPU's own inputs (teacher forcing)"""
    for l, lv in enumerate(levels):
        heads = lv["heads"]
        Q, Kw, g = store[(l, "Q")], store[(l, "Kw")], store[(l, "g")]
        ref_sub, ref_lse = oracle.modet_fwd(Q, Kw, heads, 3, want_lse=True)
        assert_close(store[(l, "sub")], ref_sub, "f32", f"iter {it} level {l} phi")
        assert_close(store[(l, "lse")], ref_lse, "f32", f"iter {it} level {l} lse")
        ref_dQ, ref_dK = oracle.modet_bwd(Q, Kw, g, heads, 3, form="gather")
        # g = diff / VN is ~1e-7 here: compare the gradients relative to their own scale
        s = float(np.abs(ref_dQ).max())
        assert_close(store[(l, "dQ")] / s, ref_dQ / s, "f32", f"iter {it} level {l} dQ")
        s = float(np.abs(ref_dK).max())
        assert_close(store[(l, "dKw")] / s, ref_dK / s, "f32", f"iter {it} level {l} dK")
        if l > 0:
            ref_w = oracle.warp(store[(l, "warp_src")], store[(l, "warp_field")], field_half_res=True)
            assert_close(store[(l, "warp_out")], ref_w, "f32", f"iter {it} level {l} warp")
            ref_c = oracle.compose(store[(l, "comp_outer")], store[(l, "comp_inner")], outer_half_res=True)
            assert_close(store[(l, "comp_out")], ref_c, "f32", f"iter {it} level {l} composition")


def test_config4_pyramid_50_iterations_teacher_forced(modet):
    """config 4 as stated: the five-level loop for a 160x192x224 pair, 50 iterations; at iterations 1, 25 and 50
    every operator call of every level (warp, forward, backward, composition) is checked against the oracle on
    the GPU's own inputs."""
    from paper_2403_16526_amd.pyramid import PyramidLoop
    levels = [dict(Q=up(l["Q"]), K=up(l["K"]), heads=l["heads"]) for l in synth.make_pyramid()]
    store = {}
    on = [False]
    loop = PyramidLoop(levels, eta=1.0,
                       record=lambda l, n, t: on[0] and store.__setitem__((l, n), t.detach().cpu().numpy()))
    losses = []
    for it in range(1, 51):
        on[0] = it in (1, 25, 50)
        store.clear()
        phi, loss = loop.iteration()
        losses.append(float(loss))
        if on[0]:
            _check_level_calls(store, levels, it)
    assert np.isfinite(losses).all() and losses[-1] < losses[0], losses
    assert phi.shape == (1, 160, 192, 224, 3)


@pytest.mark.parametrize("nlev,iters", [(4, 50), (5, 5)])
def test_config4_free_running_against_oracle_loop(modet, nlev, iters):
    """the loop run freely on both sides -- the oracle-side loop (oracle/pyramid_loop.py, plain numpy over oracle.*
    calls) and the GPU loop: all 50 iterations on the four coarser levels of config 4 (80x96x112 at the top; with
    the full-resolution level the CPU loop alone would take a few minutes), and 5 iterations on all five levels.
    Final total field and loss curve at rtol 1e-3; the observed drift is printed."""
    from paper_2403_16526_amd.pyramid import PyramidLoop
    from oracle.pyramid_loop import OraclePyramidLoop
    pyr = synth.make_pyramid()[:nlev]
    levels = [dict(Q=up(l["Q"]), K=up(l["K"]), heads=l["heads"]) for l in pyr]
    gpu_loop = PyramidLoop(levels, eta=1.0)
    cpu_loop = OraclePyramidLoop([dict(Q=l["Q"].copy(), K=l["K"], heads=l["heads"]) for l in pyr], eta=1.0)
    gl, cl = [], []
    for it in range(iters):
        phi, loss = gpu_loop.iteration()
        gl.append(float(loss))
        ref_phi, ref_loss = cpu_loop.iteration()
        cl.append(ref_loss)
    gl, cl = np.array(gl), np.array(cl)
    drift_loss = np.abs(gl - cl) / np.abs(cl)
    err = np.abs(phi.cpu().numpy().astype(np.float64) - ref_phi)
    print(f"config 4 free-running, {iters} iterations, levels 1-{nlev}: loss {cl[0]:.6f} -> {cl[-1]:.6f}; "
          f"max relative drift of the loss {drift_loss.max():.3g}; final field: max |ref| {np.abs(ref_phi).max():.3g}, "
          f"max abs difference {err.max():.3g}")
    assert drift_loss.max() <= 1e-3
    assert (err <= 1e-3 * np.abs(ref_phi) + 1e-4).all()


@pytest.mark.parametrize("name,d,heads_per_level,vol", [
    ("small", 6, (8, 4, 2, 1, 1), (160, 192, 160)),
    ("large", 12, (32, 16, 8, 4, 1), (160, 160, 192)),
])
def test_paper_model_shapes_sampled(modet, name, d, heads_per_level, vol):
    """The shapes of the paper's own models (Section 4.4: heads of 6 channels with 8, 4, 2, 1, 1 heads, heads of 12
    with 32, 16, 8, 4, 1, coarse to fine) on its two volume sizes (Section 4.1), every pyramid level: forward and
    backward with bias on the automatic kernel path (all of them tiled), sampled windows against the oracle."""
    for lvl, heads in enumerate(heads_per_level):
        D, H, W = (n >> (4 - lvl) for n in vol)
        C = d * heads
        assert modet.modet_has_tiled_kernels(C, heads, 3) == 3
        seed = 900 + 10 * lvl + (0 if name == "small" else 5)
        Q = synth.normal(seed, 0, (1, D, H, W, C))
        K = (0.8 * np.roll(Q, (1, -1, 1), axis=(1, 2, 3)) + 0.6 * synth.normal(seed, 1, (1, D, H, W, C))).astype(np.float32)
        g = synth.normal(seed, 2, (1, D, H, W, heads, 3))
        bias = (0.5 * synth.normal(seed, 3, (heads, 27))).astype(np.float32)
        Qg, Kg = up(Q), up(K)
        phi, lse = modet.modet_fwd(Qg, Kg, heads, 3, bias=up(bias), want_lse=True)
        dQ, dK = modet.modet_bwd(Qg, Kg, up(g), heads, 3, bias=up(bias), phi=phi, lse=lse)
        idx = sample_windows(1, D, H, W, heads, 3000, seed=seed, r=1)
        ref_phi, ref_lse = oracle.modet_fwd_at(Q, K, idx, heads, 3, bias=bias)
        ref_dQ, ref_dK = oracle.modet_bwd_at(Q, K, g, idx, heads, 3, bias=bias)
        t = torch.from_numpy(idx).cuda()
        tag = f"{name} model, level {lvl + 1} ({D}x{H}x{W}, C={C}, {heads} heads)"
        assert_close(phi.reshape(-1, 3)[t].cpu().numpy(), ref_phi, "f32", "phi " + tag)
        assert_close(lse.reshape(-1)[t].cpu().numpy(), ref_lse, "f32", "lse " + tag)
        assert_close(dQ.reshape(-1, d)[t].cpu().numpy(), ref_dQ, "f32", "dQ " + tag)
        assert_close(dK.reshape(-1, d)[t].cpu().numpy(), ref_dK, "f32", "dK " + tag)
        del Qg, Kg, phi, lse, dQ, dK
