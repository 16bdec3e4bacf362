"""GPU parity at randomly drawn shapes (fixed seed) for the bf16 multiclass-logistic path: the forward
contraction + softmax, sfb_apply on the fp32 array (with and without working copy) and on the two planes, and a
whole step on the planes, each against the oracle.  The draws mix arbitrary sizes with sizes at and next to the
tile edges (256 rows / columns, k-slices of 64) and, for the softmax that shares a row among several workgroups,
rows of 65536 to 200000 classes.
"""
import numpy as np
import pytest

import sfb_synth as S
from parity import TOL_BF16, TOL_F32, rel_err

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
            bound = 4 * TOL_F32 * np.sqrt(np.mean((ref - W0) ** 2)) + 2 * np.spacing(np.float32(np.max(np.abs(ref))))
            assert float(np.max(np.abs(host(W) - ref))) <= bound
        else:
            c.sfb_split_attach(W)
            U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
            Xd = dev_bf16(X)
            c.sfb_compute_sf(sfb.SFB_MLR, W, Xd, Y=dev(y), U=U)
            c.sfb_apply(W, U, Xd, 0.05)
            c.sfb_split_export(W)
            Uo, _ = oracle.mlr_sf(W0, X, y)
            ref = oracle.apply(W0.astype(np.float64), Uo, X, 0.05)
            assert rel_err(host(W) - W0, ref - W0) <= TOL_BF16
    finally:
        c.close()
