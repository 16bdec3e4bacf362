"""GPU parity at randomly drawn shapes (fixed seed).  bf16 multiclass-logistic path: the forward
contraction + softmax, sfb_apply on the fp32 array (with and without working copy) and on the two planes, and a
whole step on the planes, each against the oracle.  The draws mix arbitrary sizes with sizes at and next to the
tile edges (256 rows / columns, k-slices of 64) and, for the softmax that shares a row among several workgroups,
rows of 65536 to 200000 classes.  fp32 paths (multiclass logistic, metric learning, sparse coding, plain and
signed application): any J, D, B, drawn likewise.
"""
import numpy as np
import pytest

import sfb_synth as S
from parity import TOL_BF16, TOL_F32, dml_follow_kink, mlr_u_check, rel_err, trajectory_check

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

KINDS = ["fwd", "apply", "apply_split", "step_split", "fwd_long"]


def _cases(n, seed):
    g = np.random.default_rng(seed)
    out = []
    for case in range(n):
        kind = KINDS[case % len(KINDS)]
        if kind == "fwd_long":
            J, D, B = int(g.integers(65536 // 8, 200000 // 8)) * 8, int(g.integers(1, 20)) * 8, int(g.integers(1, 300))
        else:
            J, D, B = int(g.integers(1, 700)) * 8, int(g.integers(1, 300)) * 8, int(g.integers(1, 600))
            if g.random() < 0.3:
                J = int(g.choice([256, 512, 248, 264, 8, 1024]))
            if g.random() < 0.3:
                D = int(g.choice([64, 256, 56, 72, 8, 512, 320]))
            if g.random() < 0.3:
                B = int(g.choice([1, 63, 64, 65, 255, 256, 257, 512]))
        out.append((case, kind, J, D, B, float(g.choice([0.5, 1e-3, 1e-6])), bool(g.random() < 0.5)))
    return out


@pytest.fixture(scope="module")
def sfb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1409_5705_amd as m
    m.lib()   # raises if the HIP library is missing: no fallback
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def dev_bf16(a):
    return dev(S.bf16_bits(a)).view(torch.bfloat16)


def host(t):
    torch.cuda.synchronize()
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


@pytest.mark.parametrize("case,kind,J,D,B,eta,copy", _cases(40, seed=7))
def test_random_shape(sfb, oracle, case, kind, J, D, B, eta, copy):
    print("random shape", case, kind, J, D, B, eta, copy, flush=True)
    W0 = S.normal_matrix(J, D, 0.05, seed=100 + case)
    X, y = S.mlr_batch(J, D, B, seed=100 + case, zero_frac=0.5, bf16=True)
    c = sfb.Context(0)
    W = dev(W0)
    try:
        if kind in ("fwd", "fwd_long"):
            if copy:
                c.sfb_shadow_attach(W)
            U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
            c.sfb_compute_sf(sfb.SFB_MLR, W, dev_bf16(X), Y=dev(y), U=U)
            Uo, _ = oracle.mlr_sf(W0, X, y)
            assert rel_err(host(U), Uo) <= TOL_BF16
            mlr_u_check(host(U), Uo, y, TOL_BF16, label_tol=1e-2)
        elif kind in ("apply", "apply_split"):
            Uf = S.round_to_bf16((np.random.default_rng(case).standard_normal((B, J)) * 0.1).astype(np.float32))
            if kind == "apply_split":
                c.sfb_split_attach(W)
            elif copy:
                c.sfb_shadow_attach(W)
            c.sfb_apply(W, dev_bf16(Uf), dev_bf16(X), eta)
            if kind == "apply_split":
                c.sfb_split_export(W)
            ref = oracle.apply(W0.astype(np.float64), Uf, X, eta)
            # accumulation error of the update plus the fp32 rounding of the stored values
            trajectory_check(host(W), ref, W0, 1, TOL_F32)
        else:
            c.sfb_split_attach(W)
            U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
            Xd = dev_bf16(X)
            c.sfb_compute_sf(sfb.SFB_MLR, W, Xd, Y=dev(y), U=U)
            c.sfb_apply(W, U, Xd, 0.05)
            c.sfb_split_export(W)
            Uo, _ = oracle.mlr_sf(W0, X, y)
            mlr_u_check(host(U), Uo, y, TOL_BF16, label_tol=1e-2)
            ref = oracle.apply(W0.astype(np.float64), Uo, X, 0.05)
            assert rel_err(host(W) - W0, ref - W0) <= TOL_BF16
    finally:
        c.close()


KINDS_F32 = ["mlr", "apply", "dml", "sc", "signed"]


def _cases_f32(n, seed):
    g = np.random.default_rng(seed)
    out = []
    for case in range(n):
        kind = KINDS_F32[case % len(KINDS_F32)]
        J, D, B = int(g.integers(1, 1500)), int(g.integers(1, 1200)), int(g.integers(1, 400))
        if g.random() < 0.3:
            J = int(g.choice([64, 128, 63, 65, 256, 1, 2]))
        if g.random() < 0.3:
            D = int(g.choice([32, 64, 31, 33, 128, 1, 4]))
        if g.random() < 0.3:
            B = int(g.choice([1, 2, 63, 64, 65, 128, 129]))
        if kind == "sc":
            J, D, B = min(J, 600), min(D, 300), min(B, 100)
        out.append((case, kind, J, D, B))
    return out


@pytest.mark.parametrize("case,kind,J,D,B", _cases_f32(30, seed=11))
def test_random_shape_f32(sfb, oracle, case, kind, J, D, B):
    """The fp32 paths (no alignment requirement on J, D, B) at drawn shapes."""
    print("random shape f32", case, kind, J, D, B, flush=True)
    g = np.random.default_rng(1000 + case)
    c = sfb.Context(0)
    try:
        if kind == "mlr":
            W0 = S.normal_matrix(J, D, 0.05, seed=case)
            X, y = S.mlr_batch(J, D, B, seed=case)
            U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
            c.sfb_compute_sf(sfb.SFB_MLR, dev(W0), dev(X), Y=dev(y), U=U)
            Uo, _ = oracle.mlr_sf(W0, X, y)
            assert rel_err(host(U), Uo) <= TOL_F32
            mlr_u_check(host(U), Uo, y, TOL_F32)
        elif kind in ("apply", "signed"):
            U = g.standard_normal((B, J), dtype=np.float32)
            V = g.standard_normal((B, D), dtype=np.float32)
            W0 = S.normal_matrix(J, D, 0.01, seed=case)
            W = dev(W0)
            if kind == "apply":
                c.sfb_apply(W, dev(U), dev(V), -0.01)
                ref = oracle.apply(W0, U, V, -0.01)
            else:
                coef = g.standard_normal(B).astype(np.float32)
                c.sfb_apply_signed(W, dev(U), dev(V), dev(coef), 0.01)
                ref = oracle.apply_signed(W0, U, V, coef, 0.01)
            assert rel_err(host(W) - W0, ref - W0) <= TOL_F32
        elif kind == "dml":
            W0 = S.normal_matrix(J, D, (2.0 * J * D) ** -0.5, seed=case)      # about half the hinge terms active
            X, Y, sim = S.dml_batch(D, B, seed=case)
            U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
            V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")
            na = torch.zeros((1,), dtype=torch.int32, device="cuda:0")
            c.sfb_compute_sf(sfb.SFB_DML, dev(W0), dev(X), Y=dev(Y), sim=dev(sim), U=U, V=V, n_active=na, margin=1.0)
            Uo, Vo, no = oracle.dml_sf(W0, X, Y, sim, margin=1.0)
            Uo, no, _ = dml_follow_kink(oracle, Uo, no, host(U), W0, X, Y, sim, 1.0, 1e-5)
            assert int(host(na)[0]) == no
            assert rel_err(host(U), Uo) <= TOL_F32
            np.testing.assert_array_equal(host(V), (X - Y).astype(np.float32))
        else:
            W0 = S.sc_dictionary(J, D, seed=case)
            X = S.sc_batch(D, B, seed=case)
            U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
            V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")
            c.sfb_compute_sf(sfb.SFB_SC, dev(W0), dev(X), U=U, V=V, lam=0.1, ista_iters=20, power_iters=10)
            Uo, Vo, _ = oracle.sc_sf(W0, X, lam=0.1, ista_iters=20, power_iters=10)
            assert rel_err(host(U), Uo) <= TOL_F32
            assert rel_err(host(V), Vo) <= TOL_F32
    finally:
        c.close()
