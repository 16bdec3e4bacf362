"""Pins for the CPU oracle: things the paper and the mathematics fix, none of
which re-use the oracle's own formulas.

 * brute-force central finite differences of the stated losses (tiny, fp64);
 * closed forms and hand-worked fixtures (tests/golden);
 * library reductions (NumPy matmul, SciPy softmax, scikit-learn Lasso,
   eigvalsh);
 * algebraic invariants stated in the paper (exact reconstruction, order
   independence of the SF sum, zero-sum of the MLR factor, prox properties).
"""
import os

import numpy as np
import pytest
import scipy.special

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# Losses, written here from their definitions (not taken from the oracle).
# ----------------------------------------------------------------------------
def mlr_loss(W, X, y):
    Z = X @ W.T
    return float(np.sum(scipy.special.logsumexp(Z, axis=1) - Z[np.arange(len(y)), y]))


def dml_loss(W, X, Y, sim, margin):
    Q = (X - Y) @ W.T
    d = np.sum(Q * Q, axis=1)
    return float(np.sum(np.where(sim > 0, d, np.maximum(0.0, margin - d))))


def sc_loss_in_W(W, X, A):
    R = X - A @ W
    return 0.5 * float(np.sum(R * R))


def fd_grad(f, W, h=1e-6):
    G = np.zeros_like(W)
    for idx in np.ndindex(*W.shape):
        Wp = W.copy(); Wp[idx] += h
        Wm = W.copy(); Wm[idx] -= h
        G[idx] = (f(Wp) - f(Wm)) / (2 * h)
    return G


# ----------------------------------------------------------------------------
# 1. finite differences: sum_i u_i v_i^T is the gradient of the batch loss
# ----------------------------------------------------------------------------
def test_mlr_sf_is_gradient(oracle):
    g = np.random.default_rng(1)
    J, D, B = 5, 4, 3
    W = g.standard_normal((J, D)); X = g.standard_normal((B, D)); y = np.array([0, 4, 2])
    U, V = oracle.mlr_sf(W, X, y)
    G = fd_grad(lambda w: mlr_loss(w, X, y), W)
    np.testing.assert_allclose(U.T @ V, G, rtol=1e-6, atol=1e-8)


def test_mlr_u_is_gradient_wrt_logits(oracle):
    # u = d f / d(Wa): perturb the logits z directly.
    g = np.random.default_rng(2)
    J, D = 6, 3
    W = g.standard_normal((J, D)); x = g.standard_normal((1, D)); y = np.array([3])
    U, _ = oracle.mlr_sf(W, x, y)
    z = (W @ x[0])
    f = lambda zz: float(scipy.special.logsumexp(zz) - zz[3])
    h = 1e-6
    fd = np.array([(f(z + h * np.eye(J)[j]) - f(z - h * np.eye(J)[j])) / (2 * h) for j in range(J)])
    np.testing.assert_allclose(U[0], fd, rtol=1e-6, atol=1e-9)


def test_mlr_loss_output_matches_definition(oracle):
    g = np.random.default_rng(3)
    W = g.standard_normal((7, 5)); X = g.standard_normal((4, 5)); y = np.array([6, 0, 3, 3])
    _, _, loss = oracle.mlr_sf(W, X, y, with_loss=True)
    assert abs(loss.sum() - mlr_loss(W, X, y)) < 1e-10


def test_dml_sf_is_gradient_both_branches(oracle):
    g = np.random.default_rng(4)
    K, D, B = 3, 4, 6
    W = 0.3 * g.standard_normal((K, D))
    X = g.standard_normal((B, D)); Y = g.standard_normal((B, D))
    sim = np.array([1, 1, -1, -1, -1, -1], dtype=np.int8)
    # force one dissimilar pair far apart (inactive hinge) and one close (active)
    Y[2] = X[2] + 0.05 * g.standard_normal(D)
    Y[3] = X[3] + 50.0
    U, V, n_active, loss = oracle.dml_sf(W, X, Y, sim, margin=1.0, with_loss=True)
    d = np.sum(((X - Y) @ W.T) ** 2, axis=1)
    assert np.all(np.abs(d[sim < 0] - 1.0) > 1e-3)          # away from the kink
    assert d[2] < 1.0 < d[3]
    G = fd_grad(lambda w: dml_loss(w, X, Y, sim, 1.0), W)
    np.testing.assert_allclose(U.T @ V, G, rtol=1e-6, atol=1e-7)
    assert n_active == 2 + int(np.sum(d[2:] < 1.0))
    assert abs(loss.sum() - dml_loss(W, X, Y, sim, 1.0)) < 1e-10
    assert np.all(U[3] == 0.0)


def test_sc_sf_is_negative_gradient_in_W(oracle):
    # With the codes held fixed, d/dW 1/2||x - W^T a||^2 = -a r^T, so U^T V is the
    # *negative* gradient and the descent step is W += eta U^T V.
    g = np.random.default_rng(5)
    J, D, B = 5, 4, 3
    W = g.standard_normal((J, D)); X = g.standard_normal((B, D))
    U, V, L = oracle.sc_sf(W, X, lam=0.05, ista_iters=7, power_iters=10)
    G = fd_grad(lambda w: sc_loss_in_W(w, X, U), W)
    np.testing.assert_allclose(-(U.T @ V), G, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(V, X - U @ W, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------
# 2. hand-worked fixtures
# ----------------------------------------------------------------------------
def _rows(name):
    out = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append([float(t) for t in line.split()])
    return out


def test_mlr_hand_worked(oracle):
    W = np.array([[0.0], [np.log(3.0)]])
    for lab, u0, u1, v0, loss in _rows("mlr_hand_worked.txt"):
        U, V, l = oracle.mlr_sf(W, np.array([[1.0]]), np.array([int(lab)]), with_loss=True)
        np.testing.assert_allclose(U[0], [u0, u1], atol=1e-14)
        np.testing.assert_allclose(V[0], [v0], atol=0)
        assert abs(l[0] - loss) < 1e-14


def test_dml_hand_worked(oracle):
    W = np.array([[1.0, 0.0], [0.0, 2.0]])
    for s, x0, x1, y0, y1, u0, u1, v0, v1, loss, act in _rows("dml_hand_worked.txt"):
        U, V, n, l = oracle.dml_sf(W, np.array([[x0, x1]]), np.array([[y0, y1]]),
                                   np.array([int(s)], dtype=np.int8), margin=1.0, with_loss=True)
        np.testing.assert_allclose(U[0], [u0, u1], atol=1e-15)
        np.testing.assert_allclose(V[0], [v0, v1], atol=1e-15)
        assert n == int(act) and abs(l[0] - loss) < 1e-15


# ----------------------------------------------------------------------------
# 3. exact reconstruction and invariants of apply
# ----------------------------------------------------------------------------
def test_apply_is_sum_of_rank1_and_matmul(oracle):
    g = np.random.default_rng(6)
    N, J, D = 9, 7, 5
    W = g.standard_normal((J, D)); U = g.standard_normal((N, J)); V = g.standard_normal((N, D))
    eta = 0.37
    got = oracle.apply(W, U, V, eta)
    loop = W.copy()
    for i in range(N):
        loop -= eta * np.outer(U[i], V[i])
    np.testing.assert_allclose(got, loop, rtol=0, atol=1e-13)
    np.testing.assert_allclose(got, W - eta * (U.T @ V), rtol=0, atol=1e-13)
    # a transposed operand or swapped roles would fail this asymmetric case
    assert got.shape == (J, D)


def test_apply_invariants(oracle):
    g = np.random.default_rng(7)
    N, J, D = 12, 6, 8
    W = g.standard_normal((J, D)); U = g.standard_normal((N, J)); V = g.standard_normal((N, D))
    a = oracle.apply(W, U, V, 0.1)
    # linear in eta
    np.testing.assert_allclose(oracle.apply(a, U, V, 0.1), oracle.apply(W, U, V, 0.2), atol=1e-13)
    # additive over blocks (peer by peer == concatenated), any order of the SF rows
    b = oracle.apply(oracle.apply(W, U[:5], V[:5], 0.1), U[5:], V[5:], 0.1)
    np.testing.assert_allclose(a, b, atol=1e-13)
    p = g.permutation(N)
    np.testing.assert_allclose(a, oracle.apply(W, U[p], V[p], 0.1), atol=1e-13)
    # apply(eta) then apply(-eta) restores W
    np.testing.assert_allclose(oracle.apply(a, U, V, -0.1), W, atol=1e-13)
    # N = 0 is the identity
    np.testing.assert_array_equal(oracle.apply(W, U[:0], V[:0], 0.1), W)


# ----------------------------------------------------------------------------
# 4. MLR closed forms / library reduction
# ----------------------------------------------------------------------------
def test_apply_signed_pins(oracle):
    """Signed low-rank updates ("Low-rank Extensions", Section 2.1) against their closed forms."""
    g = np.random.default_rng(77)
    J, D = 7, 5
    W = g.standard_normal((J, D))
    # rank-2 update of a restricted Boltzmann machine: u1 v1^T - u2 v2^T
    u1, u2, v1, v2 = g.standard_normal(J), g.standard_normal(J), g.standard_normal(D), g.standard_normal(D)
    got = oracle.apply_signed(W, np.stack([u1, u2]), np.stack([v1, v2]), np.array([1.0, -1.0]), 0.3)
    assert np.allclose(got, W - 0.3 * (np.outer(u1, v1) - np.outer(u2, v2)), rtol=0, atol=1e-14)
    # rank-3 BFGS update on a square symmetric matrix: alpha u u^T - beta (u v^T + v u^T); stays symmetric
    n = 6
    H = g.standard_normal((n, n)); H = H + H.T
    u, v, alpha, beta = g.standard_normal(n), g.standard_normal(n), 0.7, 0.2
    got = oracle.apply_signed(H, np.stack([u, u, v]), np.stack([u, v, u]), np.array([alpha, -beta, -beta]), -1.0)
    want = H + alpha * np.outer(u, u) - beta * (np.outer(u, v) + np.outer(v, u))
    assert np.allclose(got, want, rtol=0, atol=1e-14)
    assert np.allclose(got, got.T, rtol=0, atol=1e-14)
    # all coefficients one: the plain SF sum; general coefficients: linear in them
    N = 9
    U, V, c = g.standard_normal((N, J)), g.standard_normal((N, D)), g.standard_normal(N)
    assert np.allclose(oracle.apply_signed(W, U, V, np.ones(N), 0.1), oracle.apply(W, U, V, 0.1), rtol=0, atol=1e-14)
    assert np.allclose(oracle.apply_signed(W, U, V, c, 0.1), W - 0.1 * (U.T * c) @ V, rtol=0, atol=1e-13)
    # a zero coefficient removes its pair; the operands are not transposed by mistake (J != D)
    c0 = c.copy(); c0[3] = 0.0
    keep = np.arange(N) != 3
    assert np.allclose(oracle.apply_signed(W, U, V, c0, 0.1), oracle.apply_signed(W, U[keep], V[keep], c[keep], 0.1),
                       rtol=0, atol=1e-14)


def test_mlr_zero_sum_and_column_sums(oracle):
    g = np.random.default_rng(8)
    J, D, B = 11, 6, 5
    W = g.standard_normal((J, D)); X = g.standard_normal((B, D)); y = g.integers(0, J, B)
    U, V = oracle.mlr_sf(W, X, y)
    np.testing.assert_allclose(U.sum(axis=1), 0.0, atol=1e-14)
    np.testing.assert_allclose((U.T @ V).sum(axis=0), 0.0, atol=1e-13)


def test_mlr_w_zero_and_shift_invariance(oracle):
    g = np.random.default_rng(9)
    J, D, B = 8, 3, 4
    X = g.standard_normal((B, D)); y = np.array([1, 7, 0, 7])
    U, _ = oracle.mlr_sf(np.zeros((J, D)), X, y)
    ref = np.full((B, J), 1.0 / J); ref[np.arange(B), y] -= 1.0
    np.testing.assert_allclose(U, ref, atol=1e-15)
    W = g.standard_normal((J, D))
    U1, _ = oracle.mlr_sf(W, X, y)
    U2, _ = oracle.mlr_sf(W + g.standard_normal((1, D)), X, y)
    np.testing.assert_allclose(U1, U2, atol=1e-13)


def test_mlr_matches_scipy_softmax_and_large_logits(oracle):
    g = np.random.default_rng(10)
    J, D, B = 9, 4, 6
    W = 300.0 * g.standard_normal((J, D)); X = g.standard_normal((B, D)); y = g.integers(0, J, B)
    U, V = oracle.mlr_sf(W, X, y)
    ref = scipy.special.softmax(X @ W.T, axis=1); ref[np.arange(B), y] -= 1.0
    assert np.all(np.isfinite(U))
    np.testing.assert_allclose(U, ref, atol=1e-12)
    np.testing.assert_array_equal(V, X)


# ----------------------------------------------------------------------------
# 5. DML closed forms
# ----------------------------------------------------------------------------
def test_dml_swap_and_identity(oracle):
    g = np.random.default_rng(11)
    D, B = 4, 5
    X = g.standard_normal((B, D)); Y = X + 0.2 * g.standard_normal((B, D))
    sim = np.array([1, -1, 1, -1, 1], dtype=np.int8)
    W = 0.5 * g.standard_normal((3, D))
    U1, V1, n1 = oracle.dml_sf(W, X, Y, sim)
    U2, V2, n2 = oracle.dml_sf(W, Y, X, sim)
    np.testing.assert_allclose(U1, -U2, atol=1e-14)
    np.testing.assert_allclose(V1, -V2, atol=1e-14)
    np.testing.assert_allclose(U1.T @ V1, U2.T @ V2, atol=1e-14)
    assert n1 == n2
    Ui, Vi, _ = oracle.dml_sf(np.eye(D), X, Y, np.ones(B, dtype=np.int8))
    np.testing.assert_allclose(Ui, 2 * (X - Y), atol=1e-14)
    np.testing.assert_allclose(Vi, X - Y, atol=1e-15)


# ----------------------------------------------------------------------------
# 6. sparse coding: closed form, library lasso, monotone objective, L bounds
# ----------------------------------------------------------------------------
def test_sc_orthonormal_rows_closed_form(oracle):
    g = np.random.default_rng(12)
    J, D, B = 4, 7, 5
    Q, _ = np.linalg.qr(g.standard_normal((D, J)))
    W = Q.T                                   # W W^T = I
    X = g.standard_normal((B, D))
    assert abs(oracle.sc_lipschitz(W, 2) - 1.0) < 1e-12
    assert abs(oracle.sc_lipschitz(W, 10) - 1.0) < 1e-12
    lam = 0.3
    T = X @ W.T
    ref = np.sign(T) * np.maximum(np.abs(T) - lam, 0.0)
    for iters in (1, 2, 20):
        U, V, L = oracle.sc_sf(W, X, lam=lam, ista_iters=iters, power_iters=10)
        np.testing.assert_allclose(U, ref, atol=1e-12)
        np.testing.assert_allclose(V, X - ref @ W, atol=1e-12)
    U0, V0, _ = oracle.sc_sf(W, X, lam=lam, ista_iters=0, power_iters=3)
    assert np.all(U0 == 0) and np.allclose(V0, X)


def test_sc_lipschitz_bounds_and_convergence(oracle):
    g = np.random.default_rng(13)
    J, D = 9, 6
    W = g.standard_normal((J, D))
    lam_max = np.linalg.eigvalsh(W.T @ W)[-1]
    Ls = [oracle.sc_lipschitz(W, k) for k in (1, 2, 5, 10, 400)]
    assert all(Ls[i] <= Ls[i + 1] + 1e-12 for i in range(len(Ls) - 1))   # non-decreasing
    assert Ls[3] <= lam_max + 1e-12
    assert abs(Ls[-1] - lam_max) < 1e-9 * lam_max
    # first application from b = 1/sqrt(D): L = ||W^T W b||
    b = np.full(D, 1 / np.sqrt(D))
    assert abs(Ls[0] - np.linalg.norm(W.T @ (W @ b))) < 1e-12


def test_sc_ista_objective_monotone_and_reaches_lasso(oracle):
    sklearn_lm = pytest.importorskip("sklearn.linear_model")
    g = np.random.default_rng(14)
    J, D, B = 6, 10, 3
    W = g.standard_normal((J, D)); X = g.standard_normal((B, D)); lam = 0.4
    L = np.linalg.eigvalsh(W @ W.T)[-1]
    obj = lambda A: 0.5 * np.sum((X - A @ W) ** 2, axis=1) + lam * np.sum(np.abs(A), axis=1)
    prev = obj(np.zeros((B, J)))
    for it in range(1, 12):
        A, _, _ = oracle.sc_sf(W, X, lam=lam, ista_iters=it, L=L)
        cur = obj(A)
        assert np.all(cur <= prev + 1e-12)
        prev = cur
    A, R, _ = oracle.sc_sf(W, X, lam=lam, ista_iters=20000, L=L)
    for i in range(B):
        # sklearn: (1/(2 n)) ||y - X w||^2 + alpha ||w||_1 with n = D "samples"
        m = sklearn_lm.Lasso(alpha=lam / D, fit_intercept=False, tol=1e-14, max_iter=200000)
        m.fit(W.T, X[i])
        np.testing.assert_allclose(A[i], m.coef_, atol=1e-7)


def test_sc_single_ista_step_by_hand(oracle):
    # one iteration from a = 0: a = soft(W x / L, lam / L)
    g = np.random.default_rng(15)
    W = g.standard_normal((4, 3)); X = g.standard_normal((2, 3)); L = 5.0; lam = 0.7
    A, R, _ = oracle.sc_sf(W, X, lam=lam, ista_iters=1, L=L)
    T = (X @ W.T) / L
    ref = np.sign(T) * np.maximum(np.abs(T) - lam / L, 0)
    np.testing.assert_allclose(A, ref, atol=1e-14)


# ----------------------------------------------------------------------------
# 7. prox
# ----------------------------------------------------------------------------
def test_prox_rows(oracle):
    g = np.random.default_rng(16)
    W = g.standard_normal((6, 5))
    W[0] *= 0.1 / np.linalg.norm(W[0])       # inside the ball
    W[1] = 0.0                               # zero row
    W[2] *= 1.0 / np.linalg.norm(W[2])       # on the sphere (up to rounding)
    P = oracle.prox_rows(W, oracle.PROX_PROJECT)
    n = np.linalg.norm(P, axis=1)
    assert np.all(n <= 1 + 1e-15)
    np.testing.assert_array_equal(P[0], W[0])
    np.testing.assert_array_equal(P[1], W[1])
    np.testing.assert_allclose(P[3:], W[3:] / np.linalg.norm(W[3:], axis=1, keepdims=True), atol=1e-15)
    np.testing.assert_allclose(oracle.prox_rows(P, oracle.PROX_PROJECT), P, atol=1e-15)   # idempotent
    Nn = oracle.prox_rows(W, oracle.PROX_NORMALIZE)
    nn = np.linalg.norm(Nn, axis=1)
    np.testing.assert_allclose(nn[[0, 2, 3, 4, 5]], 1.0, atol=1e-15)
    np.testing.assert_array_equal(Nn[1], 0.0)
    np.testing.assert_allclose(Nn[0], W[0] / np.linalg.norm(W[0]), atol=1e-15)


# ----------------------------------------------------------------------------
# 8. a full proximal-SGD step lowers the objective it claims to descend
# ----------------------------------------------------------------------------
def test_small_step_descends(oracle):
    g = np.random.default_rng(17)
    J, D, B = 6, 5, 8
    W = 0.1 * g.standard_normal((J, D)); X = g.standard_normal((B, D)); y = g.integers(0, J, B)
    U, V = oracle.mlr_sf(W, X, y)
    W1 = oracle.apply(W, U, V, 1e-3)
    assert mlr_loss(W1, X, y) < mlr_loss(W, X, y)
    Wd = g.standard_normal((J, D)); Xs = g.standard_normal((B, D))
    A, R, _ = oracle.sc_sf(Wd, Xs, lam=0.1, ista_iters=5)
    W2 = oracle.apply(Wd, A, R, -1e-3)       # W += eta U^T V
    assert sc_loss_in_W(W2, Xs, A) < sc_loss_in_W(Wd, Xs, A)


# ----------------------------------------------------------------------------
# Sparse samples / sparse second factors (Section 5: work on the non-zeros only)
# ----------------------------------------------------------------------------
def _random_csr(g, rows, cols, density, empty_rows=()):
    indptr, indices, values = [0], [], []
    for r in range(rows):
        k = 0 if r in empty_rows else int(g.binomial(cols, density))
        c = np.sort(g.choice(cols, size=k, replace=False))
        indices.extend(c.tolist())
        values.extend(g.standard_normal(k).tolist())
        indptr.append(len(indices))
    return np.array(indptr, np.int64), np.array(indices, np.int32), np.array(values, np.float64)


def test_csr_functions_pins(oracle):
    g = np.random.default_rng(4242)
    J, D, B = 9, 41, 12
    W = g.standard_normal((J, D))
    indptr, indices, values = _random_csr(g, B, D, 0.1, empty_rows=(4,))   # an empty row: its logits are all zero
    y = g.integers(0, J, size=B).astype(np.int32)
    X = np.zeros((B, D))
    for i in range(B):                           # densified by hand, not by the shared helper
        for t in range(indptr[i], indptr[i + 1]):
            X[i, indices[t]] = values[t]
    # (a) the plain definition on the dense matrix, by SciPy/NumPy
    U, loss = oracle.mlr_sf_csr(W, indptr, indices, values, y, with_loss=True)
    want = scipy.special.softmax(X @ W.T, axis=1)
    want[np.arange(B), y] -= 1.0
    assert np.allclose(U, want, rtol=0, atol=1e-14)
    assert np.allclose(loss.sum(), mlr_loss(W, X, y), rtol=1e-13)
    # an empty sample: uniform softmax minus the label
    e = np.full(J, 1.0 / J); e[y[4]] -= 1.0
    assert indptr[5] == indptr[4] and np.allclose(U[4], e, rtol=0, atol=1e-15)
    # (b) zeros add nothing: bit-identical to the dense oracle
    Ud, _ = oracle.mlr_sf(W, X, y)
    assert np.array_equal(U, Ud)
    # (c) apply: pure-Python triple loop over the stored entries
    N = B
    Uf = g.standard_normal((N, J))
    eta = 0.37
    touched = np.zeros(D, bool)
    dW = np.zeros((J, D))
    for i in range(N):
        for t in range(indptr[i], indptr[i + 1]):
            touched[indices[t]] = True
            for j in range(J):
                dW[j, indices[t]] += Uf[i, j] * values[t]
    want = W - eta * dW
    got = oracle.apply_csr(W, Uf, indptr, indices, values, eta)
    assert np.allclose(got, want, rtol=0, atol=1e-14)
    assert np.allclose(got, W - eta * Uf.T @ X, rtol=0, atol=1e-13)          # = the dense reconstruction
    assert np.array_equal(got, oracle.apply(W, Uf, X, eta))                  # zeros add nothing
    assert not touched.all() and np.array_equal(got[:, ~touched], W[:, ~touched])   # untouched columns: bit for bit
    # (d) a transposed or shifted index would show: J != D, and a single entry moves a single column
    one = oracle.apply_csr(W, Uf[:1], np.array([0, 1], np.int64), np.array([7], np.int32), np.array([2.0]), 1.0)
    diff = W - one
    assert np.allclose(diff[:, 7], 2.0 * Uf[0], rtol=0, atol=1e-15) and np.count_nonzero(np.delete(diff, 7, axis=1)) == 0
    # (e) malformed input is refused on the host
    with pytest.raises(ValueError):
        oracle.apply_csr(W, Uf[:1], np.array([0, 2], np.int64), np.array([3, 3], np.int32), np.array([1.0, 1.0]), 1.0)
    with pytest.raises(ValueError):
        oracle.apply_csr(W, Uf[:1], np.array([0, 1], np.int64), np.array([D], np.int32), np.array([1.0]), 1.0)


def test_csr_format_helpers_roundtrip():
    import sfb_synth
    X, _ = sfb_synth.mlr_batch(5, 37, 11, seed=3, zero_frac=0.8)
    indptr, indices, values = sfb_synth.csr_from_dense(X)
    assert indptr[0] == 0 and indptr[-1] == np.count_nonzero(X) == len(indices) == len(values)
    for i in range(X.shape[0]):
        seg = indices[indptr[i]:indptr[i + 1]]
        assert np.all(np.diff(seg) > 0) and np.array_equal(seg, np.nonzero(X[i])[0])
        assert np.array_equal(values[indptr[i]:indptr[i + 1]], X[i, seg])
    assert np.array_equal(sfb_synth.csr_to_dense(indptr, indices, values, X.shape[1]), X)
