"""CPU oracle for stochastic dual coordinate ascent on l2-regularised multiclass
logistic regression (Section 2.1, "Stochastic DCA"; the L2-MLR model of Section 5).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the bench's CPU
baseline, never by the product package.  Plain NumPy in fp64, slow on purpose.

Setting.  (P): min_W (1/N) sum_i f_i(W a_i) + h(W) with
    f_i(z) = log sum_j exp(z_j) - z_{y_i}          (multiclass logistic loss)
    h(W)   = (lambda / 2) ||W||_F^2                (squared l2 norm)
(D): min_U (1/N) sum_i f_i^*(-u_i) + h^*((1/N) U A^T), with the conjugates
    f_i^*(-u) = sum_j p_j log p_j,  p = onehot(y_i) - u, finite only for p in the simplex,
    h^*(Z)    = ||Z||_F^2 / (2 lambda),  so  W = grad h^*(Z) = Z / lambda,  Z = (1/N) U A^T.
The dual variable of sample i is kept as the point p_i = onehot(y_i) - u_i of the
simplex (u_i = 0, the usual start, is p_i = onehot(y_i)).

One coordinate step (the paper's three updates) on sample i:
    du_i = u_i - argmin_u { (D) with every u_j, j != i, fixed },
    u_i <- u_i - du_i,   Z <- Z - (1/N) du_i a_i^T,   W <- grad h^*(Z).
Setting the derivative of (D) along the simplex to zero gives, with z = W a_i,
c = ||a_i||^2 / (lambda N) and the current p_i,
    log p_j + c p_j = z_j + c p_{i,j} - nu   for every j,   sum_j p_j = 1,
a strictly monotone scalar equation per class inside a strictly monotone scalar
equation for nu; both are solved here by plain bisection/Newton to fp64
accuracy.  Then du_i = p - p_i.

Readings (the paper is silent or at odds with itself here):
  * the paper writes Z <- Z - du_i a_i^T; with its own definition Z = (1/N) U A^T
    the factor 1/N belongs there and is used here (callers fold it into eta);
  * a mini-batch computes every du_i at the same Z (as all SFs of a clock are
    computed at the worker's current parameters) and a common factor beta in
    (0, 1] scales all steps of the batch: u_i <- u_i - beta du_i, which keeps
    every p_i in the simplex and Z = (1/N) U A^T exact; beta = 1 with batches of
    one sample is the sequential algorithm of the text.
"""
from __future__ import annotations

import numpy as np


def dual_to_primal_l2(Z, lam):
    """W = grad h^*(Z) for h = (lam/2)||.||_F^2."""
    return np.asarray(Z, dtype=np.float64) / float(lam)


def _solve_class_equations(t, c):
    """p_j > 0 with log p_j + c p_j = t_j (vector t), by bisection in x = log p."""
    # g(x) = x + c exp(x) is increasing; g(t) >= t, and the lower end is moved down until g <= t.
    hi = np.array(t, dtype=np.float64)
    width = np.ones_like(hi)
    lo = hi - width
    while True:
        above = lo + c * np.exp(lo) > t
        if not np.any(above):
            break
        width = np.where(above, 2.0 * width, width)
        lo = np.where(above, hi - width, lo)
    for _ in range(2000):
        mid = 0.5 * (lo + hi)
        big = mid + c * np.exp(mid) > t
        hi = np.where(big, mid, hi)
        lo = np.where(big, lo, mid)
        if np.max(hi - lo) <= 1e-15 * max(1.0, float(np.max(np.abs(hi)))):
            break
    else:
        raise RuntimeError("bisection did not converge")
    return np.exp(0.5 * (lo + hi))


def coordinate_minimiser(z, p_old, c):
    """The simplex point p solving log p_j + c p_j = z_j + c p_old_j - nu, sum p = 1."""
    theta = z + c * p_old
    m = float(np.max(theta))
    lse = m + np.log(np.sum(np.exp(theta - m)))
    if c == 0.0:
        return np.exp(theta - lse)
    lo, hi = lse - c, lse                      # sum p >= 1 at lo, <= 1 at hi
    for _ in range(2000):
        nu = 0.5 * (lo + hi)
        s = float(np.sum(_solve_class_equations(theta - nu, c)))
        if s > 1.0:
            lo = nu
        else:
            hi = nu
        if hi - lo <= 1e-15 * max(1.0, abs(hi)):
            break
    else:
        raise RuntimeError("bisection did not converge")
    return _solve_class_equations(theta - 0.5 * (lo + hi), c)


def sdca_mlr_sf(W, P, X, lam, N, beta=1.0):
    """Dual steps of one mini-batch, all at the same W.

    W [J][D] primal matrix (= Z / lam), P [B][J] the batch's dual points, X [B][D]
    samples, N the number of samples in (P).  Returns (dU [B][J], P_new [B][J]):
    dU_i = beta * (p - p_i) is the first sufficient factor (the second is a_i = x_i),
    P_new = P + dU.
    """
    W = np.asarray(W, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    B, J = P.shape
    if W.shape[0] != J or X.shape != (B, W.shape[1]):
        raise ValueError("shapes: W [J][D], P [B][J], X [B][D]")
    dU = np.empty((B, J))
    for i in range(B):
        a = X[i]
        z = W @ a
        c = float(a @ a) / (float(lam) * float(N))
        p = coordinate_minimiser(z, P[i], c)
        dU[i] = float(beta) * (p - P[i])
    return dU, P + dU
