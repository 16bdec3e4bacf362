"""Seeded synthetic inputs shared by the tests, the smoke check and the bench.

This module only draws numbers: it holds none of the method's arithmetic and
imports neither the oracle nor the HIP package.  Every array is generated on the
host with ``numpy.random.default_rng`` from an explicit (seed, step, peer)
tuple, so the oracle and the GPU path are handed the very same values.

The shapes and distributions stand in for the paper's workloads (Wikipedia
tf-idf features with 325k classes; ImageNet LLC features), which are not
available: features are N(0,1), optionally with a fraction of entries zeroed
(tf-idf-like sparsity, stored dense), labels are uniform, W0 ~ N(0, sigma^2).
"""
from __future__ import annotations

import numpy as np

# Named workload shapes (classes/rows J, features D, local batch B, ...).
CONFIGS = {
    "mlr_small": dict(model="mlr", J=64, D=128, B=32, steps=10, eta=0.01, sigma=0.01),
    "mlr_peers": dict(model="mlr", J=1000, D=2048, B=256, peers=7, steps=20, eta=0.01, sigma=0.01),
    "mlr_large_bf16": dict(model="mlr", J=325000, D=10000, B=1024, steps=5, eta=0.001, sigma=0.01,
                           zero_frac=0.9, bf16=True),
    # SDCA on l2-regularised MLR at the shape of mlr_peers: local dual steps + 7 peers' factor blocks
    "sdca_peers": dict(model="sdca", J=1000, D=2048, B=256, peers=7, steps=20, lam=1e-3, n_total=100000, beta=0.125,
                       sigma=0.05),
    "dml": dict(model="dml", K=1024, D=4096, B=512, steps=10, eta=1e-4, sigma=0.01, margin=1.0),
    "sc": dict(model="sc", J=4096, D=1024, B=512, steps=5, eta=0.01, lam=0.1,
               ista_iters=20, power_iters=10),
}


def _rng(seed, *stream):
    return np.random.default_rng([int(seed)] + [int(s) for s in stream])


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits (int16 view) of fp32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    if np.any(bits & 0xFFFF):
        raise ValueError("values are not bf16-representable; call round_to_bf16 first")
    return (bits >> 16).astype(np.uint16).view(np.int16).reshape(x.shape)


def normal_matrix(rows, cols, sigma, seed, *stream):
    """rows x cols fp32 matrix ~ N(0, sigma^2)."""
    g = _rng(seed, 1000, *stream)
    return (g.standard_normal((rows, cols), dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def mlr_batch(J, D, B, seed, step=0, zero_frac=0.0, bf16=False):
    """Features X [B][D] ~ N(0,1) (a fraction zeroed, optionally bf16-rounded), labels uniform."""
    g = _rng(seed, 2000, step)
    X = g.standard_normal((B, D), dtype=np.float32)
    if zero_frac > 0.0:
        keep = g.random((B, D), dtype=np.float32) >= np.float32(zero_frac)
        X = X * keep.astype(np.float32)
    if bf16:
        X = round_to_bf16(X)
    y = g.integers(0, J, size=B, dtype=np.int64).astype(np.int32)
    return X, y


def csr_from_dense(X):
    """(indptr int64 [rows+1], indices int32 [nnz], values [nnz]) of the non-zeros of X,
    row by row with increasing column index: the same data in the sparse storage format."""
    X = np.asarray(X)
    rows, cols = np.nonzero(X)          # row-major order: rows non-decreasing, columns increasing within a row
    indptr = np.zeros(X.shape[0] + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=X.shape[0]), out=indptr[1:])
    return indptr, cols.astype(np.int32), np.ascontiguousarray(X[rows, cols])


def csr_to_dense(indptr, indices, values, cols):
    """The dense [rows][cols] array a CSR triple stores (zeros elsewhere)."""
    rows = len(indptr) - 1
    X = np.zeros((rows, cols), dtype=np.asarray(values).dtype)
    for i in range(rows):
        X[i, indices[indptr[i]:indptr[i + 1]]] = values[indptr[i]:indptr[i + 1]]
    return X


def mlr_peer_sf(J, D, n, seed, step, peer, bf16=False):
    """One simulated peer's SF block, as it would arrive over the wire.

    U [n][J]: softmax of N(0,1) logits minus the one-hot of a uniform label;
    V [n][D] ~ N(0,1).  (The softmax here is part of the input recipe, applied to
    random logits; it is not an evaluation of the model.)
    """
    g = _rng(seed, 3000, step, peer)
    logits = g.standard_normal((n, J))
    logits -= logits.max(axis=1, keepdims=True)
    e = np.exp(logits)
    U = e / e.sum(axis=1, keepdims=True)
    lab = g.integers(0, J, size=n)
    U[np.arange(n), lab] -= 1.0
    U = U.astype(np.float32)
    V = g.standard_normal((n, D), dtype=np.float32)
    if bf16:
        U = round_to_bf16(U)
        V = round_to_bf16(V)
    return U, V


def sdca_dual_points(J, y, seed, step=0, start_frac=0.25):
    """Dual points P [B][J] of SDCA on multiclass logistic regression, one simplex point per sample:
    a fraction still at its start (the one-hot vector of the label, i.e. dual variable zero), the rest
    somewhere inside the simplex (Dirichlet draws of mixed concentration), as after some epochs."""
    g = _rng(seed, 6000, step)
    B = len(y)
    P = np.empty((B, J), dtype=np.float32)
    for i in range(B):
        if g.random() < start_frac:
            P[i] = 0.0
            P[i, y[i]] = 1.0
        else:
            p = g.dirichlet(np.full(J, g.choice([0.05, 1.0, 20.0])))
            P[i] = (p / p.sum()).astype(np.float32)
    return P


def dml_batch(D, B, seed, step=0):
    """B pairs: first half similar (y = x + 0.1 N(0,1)), second half dissimilar (y ~ N(0,1))."""
    g = _rng(seed, 4000, step)
    X = g.standard_normal((B, D), dtype=np.float32)
    Y = g.standard_normal((B, D), dtype=np.float32)
    h = B // 2
    Y[:h] = X[:h] + np.float32(0.1) * Y[:h]
    sim = np.empty((B,), dtype=np.int8)
    sim[:h] = 1
    sim[h:] = -1
    return X, Y.astype(np.float32), sim


def sc_dictionary(J, D, seed):
    """J basis rows ~ N(0,1), each scaled to unit l2 norm."""
    g = _rng(seed, 5000)
    W = g.standard_normal((J, D))
    W /= np.sqrt((W * W).sum(axis=1, keepdims=True))
    return W.astype(np.float32)


def sc_batch(D, B, seed, step=0):
    g = _rng(seed, 6000, step)
    return g.standard_normal((B, D), dtype=np.float32)


def ssp_attempts(P, n, seed):
    """n seeded scheduling attempts for a simulation of P workers exchanging SF sets.

    Each attempt is ("compute", p) - worker p tries to compute its next SF set - or
    ("deliver", p, q) - the transport tries to hand worker p the next set of worker q.
    The draws know nothing of the consistency rules: whether an attempt takes effect is
    for the simulator (the library's counters on one side, the oracle on the other).
    """
    g = _rng(seed, 7000)
    out = []
    for _ in range(n):
        if P == 1 or g.random() < 0.4:
            out.append(("compute", int(g.integers(P))))
        else:
            p = int(g.integers(P))
            q = int(g.integers(P - 1))
            out.append(("deliver", p, q if q < p else q + 1))
    return out


def ssp_replay(sim, attempts):
    """Feeds a schedule of attempts (ssp_attempts) to a simulation object with compute(p) / deliver(p, q)
    methods.  A schedule is an input like the batches: the same one goes to the oracle and to the product's
    simulation; whether an attempt takes effect is decided by the object, not here."""
    for a in attempts:
        if a[0] == "compute":
            sim.compute(a[1])
        else:
            sim.deliver(a[1], a[2])


def ssp_drain(sim, P):
    """The closing schedule: round after round, every worker is offered every peer's pending sets and one more
    computation, until nothing takes effect any more."""
    progress = True
    while progress:
        progress = False
        for p in range(P):
            for q in range(P):
                if q != p:
                    while sim.deliver(p, q):
                        progress = True
            if sim.compute(p):
                progress = True
