"""Pins for the SDCA oracle (oracle/sdca.py): the dual problem (D) of Section 2.1 is
written out here from its definition, and the oracle's coordinate step is checked
against it by brute force, by a library optimiser, by the Lambert-W closed form of
the per-class equation, by weak/strong duality against the primal optimum found by
SciPy, and by the invariants the text states (Z = (1/N) U A^T, W = grad h^*(Z)).
None of this re-uses the oracle's own equations.
"""
import numpy as np
import pytest
import scipy.optimize
import scipy.special

from oracle import sdca as O


# -- (P) and (D), from the definitions ---------------------------------------
def primal(W, A, y, lam):
    Z = A @ W.T
    N = len(y)
    return float(np.mean(scipy.special.logsumexp(Z, axis=1) - Z[np.arange(N), y]) + 0.5 * lam * np.sum(W * W))


def dual(P, A, y, lam):
    """(D) as a function of the simplex points p_i = onehot(y_i) - u_i; +inf outside the simplex."""
    N, J = P.shape
    if np.any(P < 0) or np.any(np.abs(P.sum(axis=1) - 1.0) > 1e-9):
        return np.inf
    U = np.eye(J)[y] - P                                   # rows u_i
    conj = np.sum(scipy.special.xlogy(P, P))               # sum_i f_i^*(-u_i): negative entropy
    Zaux = U.T @ A / N                                     # (1/N) U A^T with U = [u_1 .. u_N] as columns
    return float(conj / N + np.sum(Zaux * Zaux) / (2.0 * lam))


def problem(seed, N=12, J=4, D=5, scale=1.0):
    g = np.random.default_rng(seed)
    A = g.standard_normal((N, D)) * scale
    y = g.integers(0, J, size=N)
    return A, y


def state(A, y, J, g):
    """A random feasible dual point and the auxiliary / primal matrices that go with it."""
    N = len(y)
    P = g.dirichlet(np.ones(J), size=N)
    U = np.eye(J)[y] - P
    return P, U.T @ A / N


@pytest.mark.parametrize("seed,lam", [(0, 0.1), (1, 1.0), (2, 0.01)])
def test_coordinate_step_minimises_the_dual(seed, lam):
    J = 4
    A, y = problem(seed, J=J)
    N = len(y)
    g = np.random.default_rng(100 + seed)
    P, Z = state(A, y, J, g)
    W = O.dual_to_primal_l2(Z, lam)
    i = 3
    dU, Pn = O.sdca_mlr_sf(W, P[i:i + 1], A[i:i + 1], lam, N, beta=1.0)
    P1 = P.copy(); P1[i] = Pn[0]
    d0, d1 = dual(P, A, y, lam), dual(P1, A, y, lam)
    assert d1 <= d0 + 1e-15
    # (a) no feasible perturbation of u_i does better, and the directional derivatives along the
    #     simplex (e_j - e_k) vanish
    for _ in range(200):
        q = g.dirichlet(np.ones(J))
        for tmix in (1e-3, 0.1, 1.0):
            P2 = P1.copy(); P2[i] = (1 - tmix) * P1[i] + tmix * q
            assert dual(P2, A, y, lam) >= d1 - 1e-14
    for j in range(J):
        for k in range(j + 1, J):
            # central difference: truncation ~ h^2 / (6 N p^2), rounding of the objective ~ 1e-13 / 2h
            h = min(1e-5, 0.01 * min(P1[i, j], P1[i, k]))
            e = np.zeros(J); e[j], e[k] = h, -h
            Pp = P1.copy(); Pp[i] += e
            Pm = P1.copy(); Pm[i] -= e
            assert abs(dual(Pp, A, y, lam) - dual(Pm, A, y, lam)) / (2 * h) < 2e-5
    # (b) a library optimiser on the same sub-problem (softmax parametrisation of the simplex)
    def sub(v):
        P2 = P.copy(); P2[i] = scipy.special.softmax(v)
        return dual(P2, A, y, lam)
    best = min((scipy.optimize.minimize(sub, g.standard_normal(J), method="BFGS", options={"gtol": 1e-12})
                for _ in range(3)), key=lambda r: r.fun)
    assert np.allclose(scipy.special.softmax(best.x), Pn[0], rtol=0, atol=1e-6)
    assert abs(best.fun - d1) < 1e-12
    # (c) the sufficient factor is the change of the dual variable, sign as in the text:
    #     u_i <- u_i - du_i  with  u_i = onehot(y_i) - p_i
    u_old = np.eye(J)[y[i]] - P[i]
    u_new = np.eye(J)[y[i]] - Pn[0]
    assert np.allclose(u_old - dU[0], u_new, rtol=0, atol=1e-15)


def test_two_class_brute_force():
    """J = 2: the sub-problem is one-dimensional; a fine grid finds its minimiser."""
    A, y = problem(7, N=6, J=2, D=3, scale=2.0)
    N, lam = len(y), 0.05
    g = np.random.default_rng(7)
    P, Z = state(A, y, 2, g)
    i = 2
    _, Pn = O.sdca_mlr_sf(O.dual_to_primal_l2(Z, lam), P[i:i + 1], A[i:i + 1], lam, N)
    grid = np.linspace(1e-9, 1 - 1e-9, 100001)
    vals = np.empty_like(grid)
    U = np.eye(2)[y] - P
    Zrest = (U.T @ A - np.outer(U[i], A[i])) / N           # (D) without sample i's term
    for n, p0 in enumerate(grid):
        p = np.array([p0, 1 - p0])
        u = np.eye(2)[y[i]] - p
        Zt = Zrest + np.outer(u, A[i]) / N
        vals[n] = np.sum(scipy.special.xlogy(p, p)) / N + np.sum(Zt * Zt) / (2 * lam)
    assert abs(grid[np.argmin(vals)] - Pn[0, 0]) < 2e-5


def test_class_equation_is_lambert_w():
    """log p + c p = t has the closed form p = W0(c e^t) / c; the p_j of a step satisfy it with one
    common shift nu, and sum to one."""
    g = np.random.default_rng(3)
    J = 9
    for c in (1e-3, 0.3, 5.0, 40.0, 150.0, 600.0):
        z = g.standard_normal(J) * 3
        p_old = g.dirichlet(np.ones(J)) if c < 100 else np.eye(J)[2]     # (large c with a one-hot point: t_j up to c)
        p = O.coordinate_minimiser(z, p_old, c)
        assert abs(p.sum() - 1.0) < 1e-13 and np.all(p > 0)
        nu = (z + c * p_old - np.log(p) - c * p)
        assert np.ptp(nu) < 1e-11                                        # one shift for all classes
        if c < 100:                                                       # (c e^t overflows beyond)
            closed = scipy.special.lambertw(c * np.exp(z + c * p_old - nu.mean())).real / c
            assert np.allclose(p, closed, rtol=1e-11, atol=0)
    # c -> 0 (a zero sample, or N -> infinity): the step goes straight to softmax(z)
    assert np.allclose(O.coordinate_minimiser(z, p_old, 0.0), scipy.special.softmax(z), rtol=1e-14)
    assert np.allclose(O.coordinate_minimiser(z, p_old, 1e-12), scipy.special.softmax(z), rtol=1e-9)


def test_fixed_point_and_beta():
    A, y = problem(5, J=5)
    N, lam, J = len(y), 0.2, 5
    g = np.random.default_rng(5)
    P, Z = state(A, y, J, g)
    W = O.dual_to_primal_l2(Z, lam)
    # a dual point that already equals softmax(W a_i) is optimal for its coordinate: no step
    i = 1
    P[i] = scipy.special.softmax(W @ A[i])        # (changes Z's definition, but the step only sees W and p_i)
    dU, Pn = O.sdca_mlr_sf(W, P[i:i + 1], A[i:i + 1], lam, N)
    assert np.max(np.abs(dU)) < 1e-13
    # beta scales the step; the result stays in the simplex
    dU1, _ = O.sdca_mlr_sf(W, P, A, lam, N, beta=1.0)
    dUh, Ph = O.sdca_mlr_sf(W, P, A, lam, N, beta=0.25)
    assert np.allclose(dUh, 0.25 * dU1, rtol=0, atol=1e-15)
    assert np.all(Ph >= 0) and np.allclose(Ph.sum(axis=1), 1.0, atol=1e-13)
    assert np.allclose(dU1.sum(axis=1), 0.0, atol=1e-13)                 # factors sum to zero over classes


def test_sequential_sdca_reaches_the_primal_optimum(oracle):
    """Batches of one sample, beta = 1 (the algorithm of the text): the dual objective never increases,
    P(W) + D(U) >= 0 throughout (weak duality; (D) is written as a minimisation) and goes to zero, and W
    converges to the minimiser of (P) found by SciPy.  Z is kept by rank-1 updates and stays (1/N) U A^T."""
    J, D, N, lam = 3, 4, 10, 0.1
    A, y = problem(11, N=N, J=J, D=D)
    P = np.eye(J)[y].astype(np.float64)                                   # u_i = 0
    Z = np.zeros((J, D))
    g = np.random.default_rng(11)
    last = dual(P, A, y, lam)
    for it in range(60 * N):
        i = int(g.integers(0, N))
        W = O.dual_to_primal_l2(Z, lam)
        dU, Pn = O.sdca_mlr_sf(W, P[i:i + 1], A[i:i + 1], lam, N)
        P[i] = Pn[0]
        Z = oracle.apply(Z, dU, A[i:i + 1], 1.0 / N)                      # Z <- Z - (1/N) du_i a_i^T
        now = dual(P, A, y, lam)
        assert now <= last + 1e-13
        last = now
        if it % 50 == 0:
            assert primal(O.dual_to_primal_l2(Z, lam), A, y, lam) + now >= -1e-12
    U = np.eye(J)[y] - P
    assert np.allclose(Z, U.T @ A / N, rtol=0, atol=1e-13)
    W = O.dual_to_primal_l2(Z, lam)
    assert primal(W, A, y, lam) + last < 1e-9                             # duality gap closed
    best = scipy.optimize.minimize(lambda w: primal(w.reshape(J, D), A, y, lam), np.zeros(J * D), method="BFGS",
                                   options={"gtol": 1e-10})
    assert np.allclose(W, best.x.reshape(J, D), rtol=0, atol=1e-5)
    # at the optimum the dual points are the model's class probabilities
    assert np.allclose(P, scipy.special.softmax(A @ W.T, axis=1), rtol=0, atol=1e-5)


def test_minibatch_keeps_the_invariants(oracle):
    """A mini-batch at a common W with beta = 1/B: the dual still decreases (convex combination of
    coordinate minimisers) and Z = (1/N) U A^T holds after the rank-1 updates."""
    J, D, N, lam, B = 5, 6, 16, 0.05, 4
    A, y = problem(13, N=N, J=J, D=D)
    P = np.eye(J)[y].astype(np.float64)
    Z = np.zeros((J, D))
    last = dual(P, A, y, lam)
    for step in range(40):
        idx = np.arange(step * B, step * B + B) % N
        W = O.dual_to_primal_l2(Z, lam)
        dU, Pn = O.sdca_mlr_sf(W, P[idx], A[idx], lam, N, beta=1.0 / B)
        P[idx] = Pn
        Z = oracle.apply(Z, dU, A[idx], 1.0 / N)
        now = dual(P, A, y, lam)
        assert now <= last + 1e-13
        last = now
    assert np.allclose(Z, (np.eye(J)[y] - P).T @ A / N, rtol=0, atol=1e-13)
