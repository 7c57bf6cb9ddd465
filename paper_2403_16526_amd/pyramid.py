"""Coarse-to-fine driver of the five-level pairwise-optimisation loop (paper Section 3.1, Fig. 2):
per level, warp the moving features by the 2x-upsampled accumulated field, run the ModeT operator
forward and backward, compose the fields.

The paper optimises network weights through the whole registration network; the encoder, RegHead and
loss are outside this library, so this driver is a stand-in that exercises the same operator calls on
the same shapes: the per-level query features are the free variables, the sub-fields are fused by a
plain mean over heads, the loss is 0.5*mean|sub - target|^2 and the update is plain gradient descent.
All operator work goes through libmodet: warp, forward, backward, and the composition with the coarser
level's field (upsampled inside the library).  What is left in torch is the stand-in for the parts of the
network this library does not contain: the mean over heads, the loss and the update.
"""
from __future__ import annotations

import torch

from . import modet


class PyramidLoop:
    def __init__(self, levels, targets=None, eta: float = 1.0, k: int = 3, record=None, timer=None):
        """levels: list of dicts with Q, K (GPU tensors [1,D,H,W,C]) and heads, coarse to fine."""
        self.levels = levels
        self.targets = targets
        self.eta = eta
        self.k = k
        self.record = record          # optional callable(level, name, tensor) for teacher-forced checks
        self.timer = timer            # optional callable(level, name, fn) -> fn(): times one library call

    def _rec(self, l, name, t):
        if self.record is not None:
            self.record(l, name, t)

    def _call(self, l, name, fn):
        return fn() if self.timer is None else self.timer(l, name, fn)

    def iteration(self):
        """One pass over all levels; returns the finest total field and the summed loss (a GPU scalar)."""
        phi_prev = None
        loss = None
        for l, lv in enumerate(self.levels):
            Q, K, heads = lv["Q"], lv["K"], lv["heads"]
            if phi_prev is None:
                Kw = K
            else:
                self._rec(l, "warp_src", K)
                self._rec(l, "warp_field", phi_prev)
                Kw = self._call(l, "warp", lambda: modet.modet_warp(K, phi_prev, field_half_res=True))
                self._rec(l, "warp_out", Kw)
            sub, lse = self._call(l, "fwd", lambda: modet.modet_fwd(Q, Kw, heads, self.k, want_lse=True))
            varphi = sub.mean(dim=4) if heads > 1 else sub.view(sub.shape[:4] + (3,))
            if phi_prev is None:
                phi = varphi
            else:
                # phi_l(p) = varphi(p) + up(p + varphi(p)), up = the 2x upsampled field of the level below
                phi = self._call(l, "compose", lambda: modet.modet_compose(phi_prev, varphi, outer_half_res=True))
                for name, t in (("comp_outer", phi_prev), ("comp_inner", varphi), ("comp_out", phi)):
                    self._rec(l, name, t)
            diff = sub if self.targets is None else sub - self.targets[l]
            nvn = sub.numel() // 3
            g = diff * (1.0 / nvn)
            dQ, dKw = self._call(l, "bwd", lambda: modet.modet_bwd(Q, Kw, g, heads, self.k, phi=sub, lse=lse))
            for name, t in (("Q", Q), ("Kw", Kw), ("g", g), ("sub", sub), ("lse", lse), ("dQ", dQ), ("dKw", dKw)):
                self._rec(l, name, t)
            # dKw would go back through the warp's adjoint to the un-warped features; the stand-in drops it
            Q.add_(dQ, alpha=-self.eta * nvn)      # step on the un-normalised gradient so that phi moves visibly
            li = torch.linalg.vector_norm(diff).square() * (0.5 / diff.numel())
            loss = li if loss is None else loss + li
            phi_prev = phi
        return phi_prev, loss
