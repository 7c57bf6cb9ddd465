"""The library's calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no memset),
so a sequence of them can be captured into a HIP graph and replayed: the coarse pyramid levels, where a call takes
tens of microseconds, are bound by launch overhead otherwise.  Every replay is checked against the eager result
for the data the static buffers hold at that moment, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2403_16526_amd import synth
from parity_util import up

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def modet():
    assert torch.cuda.is_available(), "needs the MI355X"
    from paper_2403_16526_amd import modet as m
    return m


def test_captured_level_replays_like_eager(modet):
    B, D, H, W, C, heads, k = 1, 20, 24, 28, 32, 4, 3          # a coarse pyramid level
    dev = "cuda"
    f32 = dict(device=dev, dtype=torch.float32)
    Q, K = torch.empty((B, D, H, W, C), **f32), torch.empty((B, D, H, W, C), **f32)
    g = torch.empty((B, D, H, W, heads, 3), **f32)
    coarse = torch.empty((B, D // 2, H // 2, W // 2, 3), **f32)
    bias = up((0.3 * synth.normal(91, 0, (heads, k ** 3))).astype(np.float32))
    Kw = torch.empty_like(K)
    phi, lse = torch.empty((B, D, H, W, heads, 3), **f32), torch.empty((B, D, H, W, heads), **f32)
    dQ, dK = torch.empty_like(Q), torch.empty_like(Q)
    ws = torch.empty(modet.modet_bwd_workspace_bytes(B, D, H, W, C, heads, k, have_stats=True, want_dbias=True),
                     device=dev, dtype=torch.uint8)
    total = torch.empty((B, D, H, W, 3), **f32)
    varphi = torch.empty((B, D, H, W, 3), **f32)

    def load(seed):
        Q.copy_(up(synth.normal(seed, 0, tuple(Q.shape))))
        K.copy_(up(synth.normal(seed, 1, tuple(K.shape))))
        g.copy_(up(synth.normal(seed, 2, tuple(g.shape))))
        coarse.copy_(up(synth.smooth_real_field(seed, B, D // 2, H // 2, W // 2, 1.0)))
        varphi.copy_(up(synth.smooth_real_field(seed + 1, B, D, H, W, 0.7)))

    def level():
        modet.modet_warp(K, coarse, field_half_res=True, out=Kw)
        modet.modet_fwd(Q, Kw, heads, k, bias=bias, out=(phi, lse))
        res = modet.modet_bwd(Q, Kw, g, heads, k, bias=bias, phi=phi, lse=lse, want_dbias=True, out=(dQ, dK),
                              workspace=ws)
        modet.modet_compose(varphi, varphi, out=total)
        return res[2]

    load(100)
    db_eager = level()                       # warm-up outside the capture (first-launch queries happen here)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        level()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        db_graph = level()

    for seed in (101, 102, 103):
        load(seed)
        db_eager = level().clone()
        want = [t.clone() for t in (Kw, phi, lse, dQ, dK, total)]
        torch.cuda.synchronize()
        for t in (Kw, phi, lse, dQ, dK, total, db_graph):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("Kw", "phi", "lse", "dQ", "dK", "total"), (Kw, phi, lse, dQ, dK, total), want):
            assert torch.equal(a, b), f"replay differs from eager in {name} (seed {seed})"
        # the bias gradient's fp64 sums are added in no fixed order: equal after rounding to fp32 in practice
        assert torch.allclose(db_graph, db_eager, rtol=1e-6, atol=1e-7), f"dbias (seed {seed})"
