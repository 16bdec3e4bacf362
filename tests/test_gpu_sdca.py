"""GPU parity of the SDCA entry points (dual coordinate steps of l2-regularised
multiclass logistic regression, Section 2.1) against oracle/sdca.py."""
import numpy as np
import pytest

import sfb_synth as S
from parity import TOL_F32, rel_err
from parity import trajectory_check as _trajectory_check

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sfb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1409_5705_amd as m
    m.lib()   # raises if the HIP library is missing: no fallback
    return m


@pytest.fixture(scope="module")
def ctx(sfb):
    c = sfb.Context(0)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


@pytest.mark.parametrize("J,D,B,lam,N,beta,sigma", [
    (64, 128, 32, 0.1, 1000, 1.0, 0.3),            # c ~ 1
    (1000, 2048, 256, 1e-3, 100000, 0.25, 0.05),   # c ~ 20: strongly coupled class equations
    (1000, 2048, 64, 0.1, 1000000, 1.0, 0.05),     # c ~ 0.02: close to a plain softmax
    (37, 50, 7, 0.01, 500, 0.5, 0.5),              # nothing aligned
    (5000, 264, 40, 1e-4, 20000, 1.0, 0.02),       # c ~ 130, many classes per thread
])
def test_sdca_mlr_sf(ctx, sfb, J, D, B, lam, N, beta, sigma):
    from oracle import sdca as O
    print("sdca_mlr_sf", J, D, B, lam, N, beta, flush=True)
    W0 = S.normal_matrix(J, D, sigma, seed=8)
    X, y = S.mlr_batch(J, D, B, seed=8)
    X[B // 2] = 0.0                                 # a zero sample: c = 0
    P0 = S.sdca_dual_points(J, y, seed=8)
    P = dev(P0)
    dU = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    ctx.sfb_sdca_mlr_sf(dev(W0), dev(X), P, lam, N, beta, dU)
    dUo, Po = O.sdca_mlr_sf(W0, P0, X, lam, N, beta)
    e1, e2 = rel_err(host(dU), dUo), rel_err(host(P), Po)
    print("  err dU %.3g  P %.3g" % (e1, e2), flush=True)
    assert e1 <= TOL_F32 and e2 <= TOL_F32
    Pg, dUg = host(P), host(dU)
    assert np.all(Pg >= 0) and np.max(np.abs(Pg.sum(axis=1) - 1.0)) < 1e-5
    assert np.max(np.abs(dUg.sum(axis=1))) < 1e-5
    assert np.array_equal(Pg, P0 + dUg)             # P is advanced by exactly the factor that is sent


def test_sdca_trajectory(ctx, sfb, oracle):
    """Mini-batch SDCA from the start (u = 0, Z = 0): SF computation, application to Z with eta = 1/N,
    W = Z / lambda, several passes; against the oracle's trajectory, and against the shortcut that applies
    the factors to W directly with eta = 1 / (lambda N)."""
    from oracle import sdca as O
    J, D, N, B, lam, steps = 100, 264, 512, 128, 0.01, 8
    beta = 0.5
    A, y = S.mlr_batch(J, D, N, seed=9)
    P0 = np.eye(J, dtype=np.float32)[y]
    Pg, Zg, Wg = dev(P0), torch.zeros((J, D), device="cuda:0"), torch.zeros((J, D), device="cuda:0")
    Ws = torch.zeros((J, D), device="cuda:0")       # shortcut replica
    Ad = dev(A)
    Po, Zo = P0.astype(np.float64), np.zeros((J, D))
    dU = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    for step in range(steps):
        idx = np.arange(step * B, step * B + B) % N
        it = torch.from_numpy(idx).to("cuda:0")
        Pb = Pg[it].contiguous()
        Xb = Ad[it].contiguous()
        ctx.sfb_sdca_mlr_sf(Wg, Xb, Pb, lam, N, beta, dU)
        Pg[it] = Pb
        ctx.sfb_apply(Zg, dU, Xb, 1.0 / N)
        ctx.sfb_dual_to_primal_l2(Zg, Wg, lam)
        ctx.sfb_apply(Ws, dU, Xb, 1.0 / (lam * N))
        dUo, Pn = O.sdca_mlr_sf(O.dual_to_primal_l2(Zo, lam), Po[idx], A[idx], lam, N, beta)
        Po[idx] = Pn
        Zo = oracle.apply(Zo, dUo, A[idx], 1.0 / N)
    Wo = O.dual_to_primal_l2(Zo, lam)
    _trajectory_check(host(Wg), Wo, np.zeros((J, D)), steps, TOL_F32)
    _trajectory_check(host(Zg), Zo, np.zeros((J, D)), steps, TOL_F32)
    e_p = rel_err(host(Pg), Po)
    print('  sdca trajectory: P err %.3g' % e_p, flush=True)
    assert e_p <= TOL_F32
    assert rel_err(host(Ws), host(Wg)) <= 1e-5
    # Z = (1/N) U A^T with u_i = onehot(y_i) - p_i still holds on the GPU's own state
    Ug = np.eye(J)[y] - host(Pg).astype(np.float64)
    e_z = rel_err(host(Zg), Ug.T @ A.astype(np.float64) / N)
    print('  sdca trajectory: Z invariant err %.3g' % e_z, flush=True)
    assert e_z <= TOL_F32


def test_sdca_rejects_bad_arguments(ctx, sfb):
    J, D, B = 16, 24, 4
    W = torch.zeros((J, D), device="cuda:0"); X = torch.zeros((B, D), device="cuda:0")
    P = torch.full((B, J), 1.0 / J, device="cuda:0"); dU = torch.empty((B, J), device="cuda:0")
    for lam, N, beta in ((0.0, 10, 1.0), (-1.0, 10, 1.0), (0.1, 0, 1.0), (0.1, 10, 0.0), (0.1, 10, 1.5)):
        with pytest.raises(sfb.SfbError) as e:
            ctx.sfb_sdca_mlr_sf(W, X, P, lam, N, beta, dU)
        assert e.value.code == sfb.SFB_EINVAL
    with pytest.raises(sfb.SfbError):
        ctx.sfb_dual_to_primal_l2(W, W, 0.0)
    # all-zero samples at W = 0: every dual point goes to the uniform distribution
    ctx.sfb_sdca_mlr_sf(W, X, P, 0.1, 10, 1.0, dU)
    torch.cuda.synchronize()
    assert float(dU.abs().max()) < 1e-7
