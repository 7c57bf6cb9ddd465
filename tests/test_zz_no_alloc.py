"""modet_bwd_static (the entry point that allocates nothing) against modet_bwd, through the C ABI."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(shape, heads, k, seed):
    from paper_2403_16526_amd import synth
    B, D, H, W, C = shape
    c = synth.make_case(B, D, H, W, C, heads, k, keys="displaced", m=1, seed=seed)
    bias = (0.3 * synth.normal(seed + 1, 5, (heads, k ** 3))).astype(np.float32)
    return [torch.from_numpy(c[n]).cuda() for n in ("Q", "K", "dphi")] + [torch.from_numpy(bias).cuda()]


def test_static_scratch_backward_matches_modet_bwd_twice_in_a_row():
    from paper_2403_16526_amd import modet
    # two calls in a row on the same GPU, the second on a smaller input: what the first one left in the
    # built-in scratch must not leak into the second.  Both use the scratch for the recomputed statistics and
    # for the sums of the bias gradient; then once more with the forward's statistics handed over.
    for shape, heads, k, seed in (((1, 20, 30, 70, 16), 2, 3, 41), ((1, 9, 11, 35, 8), 1, 3, 42)):
        Q, K, g, bias = _case(shape, heads, k, seed)
        want_dQ, want_dK, want_db = modet.modet_bwd(Q, K, g, heads, k, bias=bias, want_dbias=True)
        dQ, dK = torch.full_like(want_dQ, float("nan")), torch.full_like(want_dK, float("nan"))
        db = torch.full_like(want_db, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        modet.modet_bwd_static(Q, K, g, heads, k, (dQ, dK), bias=bias, dbias=db)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        # the same kernels on the same inputs: dQ and dK bit for bit; the bias gradient's fp64 sums are added
        # in an order that is not fixed, so it is compared at fp32 rounding
        assert torch.equal(dQ, want_dQ) and torch.equal(dK, want_dK)
        scale = float(want_db.abs().max())
        assert float((db - want_db).abs().max()) <= 1e-6 * scale
        phi, lse = modet.modet_fwd(Q, K, heads, k, bias=bias, want_lse=True)
        dQ.fill_(float("nan")); dK.fill_(float("nan"))
        modet.modet_bwd_static(Q, K, g, heads, k, (dQ, dK), bias=bias, phi=phi, lse=lse)
        ref_dQ, ref_dK = modet.modet_bwd(Q, K, g, heads, k, bias=bias, phi=phi, lse=lse)
        assert torch.equal(dQ, ref_dQ) and torch.equal(dK, ref_dK)


def test_static_scratch_backward_rejects_what_does_not_fit():
    from paper_2403_16526_amd import modet
    Q = torch.zeros((1, 64, 64, 129, 8), device="cuda")
    g = torch.zeros((1, 64, 64, 129, 1, 3), device="cuda")
    dQ, dK = torch.empty_like(Q), torch.empty_like(Q)
    with pytest.raises(modet.ModetError) as e:
        modet.modet_bwd_static(Q, Q, g, 1, 3, (dQ, dK))
    assert e.value.status == -5
    # with the statistics passed in nothing but the bias gradient needs scratch: the same shape is accepted
    phi, lse = modet.modet_fwd(Q, Q, 1, 3, want_lse=True)
    modet.modet_bwd_static(Q, Q, g, 1, 3, (dQ, dK), phi=phi, lse=lse)
    torch.cuda.synchronize()
    assert float(dQ.abs().max()) == 0.0 and float(dK.abs().max()) == 0.0      # zero upstream gradient
