"""Oracle-side twin of the coarse-to-fine loop (paper Section 3.1) -- TEST INFRASTRUCTURE ONLY.

The same steps as the GPU driver of the five-level pairwise-optimisation loop, in plain numpy over the oracle's
own functions: per level, warp the moving features by the upsampled total field of the level below, forward,
mean over heads, composition with that field, backward, plain gradient step on the query features (a stand-in
for the parts of the network outside the operator).  Imports nothing of the GPU path.  Parity unpinned: the loop
is a stand-in of this build's own definition; every function it calls is pinned on its own."""
import numpy as np

import oracle


class OraclePyramidLoop:
    def __init__(self, levels, targets=None, eta=1.0, k=3):
        """levels: dicts with Q, K (numpy fp32 [1,D,H,W,C]) and heads, coarse to fine; Q is updated in place."""
        self.levels, self.targets, self.eta, self.k = levels, targets, eta, k

    def iteration(self):
        phi_prev, loss = None, 0.0
        for l, lv in enumerate(self.levels):
            Q, K, heads = lv["Q"], lv["K"], lv["heads"]
            # the moving features deformed by the upsampled total field of the level below (an fp32 tensor, as
            # every tensor that goes from one call to the next)
            Kw = K if phi_prev is None else oracle.warp(K, phi_prev, field_half_res=True).astype(np.float32)
            sub = oracle.modet_fwd(Q, Kw, heads, self.k).astype(np.float32)
            varphi = sub.astype(np.float64).mean(axis=4).astype(np.float32)          # equal-weight fusion of the heads
            phi = varphi if phi_prev is None else oracle.compose(phi_prev, varphi, outer_half_res=True).astype(np.float32)
            tgt = 0.0 if self.targets is None else self.targets[l]
            diff = sub.astype(np.float64) - tgt
            nvn = sub.size // 3
            g = (diff * (1.0 / nvn)).astype(np.float32)
            dQ, _ = oracle.modet_bwd(Q, Kw, g, heads, self.k, form="gather")
            Q -= (self.eta * nvn * dQ).astype(np.float32)
            loss += 0.5 * float((diff * diff).mean())
            phi_prev = phi
        return phi_prev.astype(np.float64), loss
