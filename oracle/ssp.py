"""CPU oracle of SF application under BSP / SSP / ASP (TEST INFRASTRUCTURE ONLY).

Follows Section 4 ("SSP-SFB") and the local update rule Eq. (1) of Section 5 in
the paper's notation: t[p] is the number of SF sets worker p has computed,
tau[p][q] the number of sets of q that p has received and applied, s the
staleness bound.  A worker pauses while t_p - tau_p^q > s for some q; it never
uses a set of q that is ahead of its own iteration count (tau_p^q <= t_p); its
replica is W^0 plus every update it has applied (its own at once, the peers' in
the order they were produced).  All arithmetic in fp64 through the plain
oracle functions.  Shares no code with the product.
"""
from __future__ import annotations

import numpy as np

from . import apply as oracle_apply
from . import mlr_sf as oracle_mlr_sf


class SspOracle:
    def __init__(self, P, s, W0, eta, batch_fn, T):
        """batch_fn(p, t) -> (X, y): the mini-batch worker p uses for its set t; T sets per worker at most."""
        self.P, self.s, self.eta, self.T = P, s, eta, T
        self.W = [np.array(W0, dtype=np.float64) for _ in range(P)]
        self.t = [0] * P
        self.tau = [[0] * P for _ in range(P)]
        self.arrived = [[0] * P for _ in range(P)]
        self.sets = {}            # (q, t) -> (U, V)
        self.batch_fn = batch_fn
        self.trace = []           # effective events
        self.max_stale = 0

    # --- rules -----------------------------------------------------------------
    def may_compute(self, p):
        if self.t[p] >= self.T:
            return False
        if self.s < 0:
            return True
        return all(self.t[p] - self.tau[p][q] <= self.s for q in range(self.P) if q != p)

    def _apply_ready(self, p):
        while True:
            ready = [(self.tau[p][q], q) for q in range(self.P)
                     if q != p and self.tau[p][q] < self.arrived[p][q] and self.tau[p][q] < self.t[p]]
            if not ready:
                return
            t, q = min(ready)
            U, V = self.sets[(q, t)]
            self.W[p] = oracle_apply(self.W[p], U, V, self.eta)
            self.tau[p][q] += 1
            self.trace.append(("apply", p, q, t))

    # --- events ----------------------------------------------------------------
    def compute(self, p):
        if not self.may_compute(p):
            return False
        for q in range(self.P):
            if q != p:
                self.max_stale = max(self.max_stale, self.t[p] - self.tau[p][q])
        X, y = self.batch_fn(p, self.t[p])
        U, _ = oracle_mlr_sf(self.W[p], X, y)
        V = np.asarray(X, dtype=np.float64)
        self.sets[(p, self.t[p])] = (U, V)
        self.W[p] = oracle_apply(self.W[p], U, V, self.eta)
        self.trace.append(("compute", p, self.t[p]))
        self.t[p] += 1
        self._apply_ready(p)
        return True

    def deliver(self, p, q):
        if self.arrived[p][q] >= self.t[q]:
            return False
        self.trace.append(("deliver", p, q, self.arrived[p][q]))
        self.arrived[p][q] += 1
        self._apply_ready(p)
        return True
