"""Coarse-to-fine driver of the five-level pairwise-optimisation loop (paper Section 3.1, Fig. 2):
per level, warp the moving features by the 2x-upsampled accumulated field, run the ModeT operator
forward and backward, compose the fields.

The paper optimises network weights through the whole registration network; the encoder, RegHead and
loss are outside this library, so this driver is a stand-in that exercises the same operator calls on
the same shapes: the per-level query features are the free variables, the sub-fields are fused by a
plain mean over heads, the loss is 0.5*mean|sub - target|^2 and the update is plain gradient descent.
All operator work goes through libmodet; the glue (mean, axpy, 2x field upsampling for the
composition) is a handful of torch ops.
"""
from __future__ import annotations

import torch
import torch.nn.functional as F

from . import modet


def upsample_field(phi_c: torch.Tensor) -> torch.Tensor:
    """[B,Dc,Hc,Wc,3] -> [B,2Dc,2Hc,2Wc,3], trilinear with half-voxel centres, values doubled."""
    x = phi_c.permute(0, 4, 1, 2, 3)
    x = F.interpolate(x, scale_factor=2, mode="trilinear", align_corners=False)
    return (2.0 * x).permute(0, 2, 3, 4, 1).contiguous()


class PyramidLoop:
    def __init__(self, levels, targets=None, eta: float = 1.0, k: int = 3, record=None):
        """levels: list of dicts with Q, K (GPU tensors [1,D,H,W,C]) and heads, coarse to fine."""
        self.levels = levels
        self.targets = targets
        self.eta = eta
        self.k = k
        self.record = record          # optional callable(level, name, tensor) for teacher-forced checks

    def _rec(self, l, name, t):
        if self.record is not None:
            self.record(l, name, t)

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
                Kw = modet.modet_warp(K, phi_prev, field_half_res=True)
                self._rec(l, "warp_out", Kw)
            sub, lse = modet.modet_fwd(Q, Kw, heads, self.k, want_lse=True)
            varphi = sub.mean(dim=4)
            if phi_prev is None:
                phi = varphi
            else:
                up = upsample_field(phi_prev)
                phi = modet.modet_compose(up, varphi)            # phi_l(p) = varphi(p) + up(p + varphi(p))
                for name, t in (("comp_outer", up), ("comp_inner", varphi), ("comp_out", phi)):
                    self._rec(l, name, t)
            tgt = 0.0 if self.targets is None else self.targets[l]
            diff = sub - tgt
            nvn = sub.numel() // 3
            g = (diff / nvn).contiguous()
            dQ, dKw = modet.modet_bwd(Q, Kw, g, heads, self.k, phi=sub, lse=lse)
            for name, t in (("Q", Q), ("Kw", Kw), ("g", g), ("sub", sub), ("lse", lse), ("dQ", dQ), ("dKw", dKw)):
                self._rec(l, name, t)
            lv["dKw_checksum"] = dKw.double().sum()
            Q.sub_(self.eta * nvn * dQ)      # step on the un-normalised gradient so that phi moves visibly
            li = 0.5 * (diff * diff).mean()
            loss = li if loss is None else loss + li
            phi_prev = phi
        return phi_prev, loss
