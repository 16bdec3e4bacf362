"""P workers with one replica of W each, simulated on one GPU (multiclass logistic regression).

Host orchestration only: the SF sets are computed and applied by the library's kernels
(sfb_compute_sf, sfb_apply) and the consistency rules of Section 4 ("SSP-SFB") / Eq. (1) of
Section 5 are the library's counters (sfb_ssp_*, include/sfb_ssp.h).  The "transport" is a
dictionary of device buffers; an SF set is dropped once every peer has applied it.
"""
from __future__ import annotations

import torch

from .binding import SFB_MLR, Context, SspClock


class SspSimulation:
    def __init__(self, ctx: Context, P: int, s: int, W0: torch.Tensor, eta: float, batch_fn, T: int):
        """batch_fn(p, t) -> (X, y) device tensors of worker p's mini-batch for its set t; at most T sets each."""
        self.ctx, self.P, self.s, self.eta, self.T = ctx, P, s, float(eta), T
        self.W = [W0.clone() for _ in range(P)]
        self.clock = SspClock(P, s)
        self.sets = {}      # (q, t) -> [U, V, peers still to apply it]
        self.batch_fn = batch_fn
        self.trace = []

    def _apply_ready(self, p):
        while True:
            nxt = self.clock.sfb_ssp_pop_apply(p)
            if nxt is None:
                return
            q, t = nxt
            ent = self.sets[(q, t)]
            self.ctx.sfb_apply(self.W[p], ent[0], ent[1], self.eta)
            self.trace.append(("apply", p, q, t))
            ent[2] -= 1
            if ent[2] == 0:
                del self.sets[(q, t)]

    def compute(self, p) -> bool:
        if self.clock.sfb_ssp_clock(p) >= self.T or not self.clock.sfb_ssp_can_compute(p):
            return False
        t = self.clock.sfb_ssp_clock(p)
        X, y = self.batch_fn(p, t)
        J = self.W[p].shape[0]
        U = torch.empty((X.shape[0], J), dtype=X.dtype, device=X.device)
        self.ctx.sfb_compute_sf(SFB_MLR, self.W[p], X, Y=y, U=U)
        if self.P > 1:
            self.sets[(p, t)] = [U, X, self.P - 1]
        self.ctx.sfb_apply(self.W[p], U, X, self.eta)
        got = self.clock.sfb_ssp_computed(p)
        assert got == t
        self.trace.append(("compute", p, t))
        self._apply_ready(p)
        return True

    def deliver(self, p, q) -> bool:
        if self.clock.sfb_ssp_arrived(p, q) >= self.clock.sfb_ssp_clock(q):
            return False
        t = self.clock.sfb_ssp_delivered(p, q)
        self.trace.append(("deliver", p, q, t))
        self._apply_ready(p)
        return True
