"""GPU parity: the HIP path (through the C-ABI) against the CPU oracle, element
by element, on the same seeded inputs.  Sizes span several tiles plus ragged
tails; the edge cases (empty batch, unaligned shapes, hinge ties) are included.

Tolerances (see tests/parity.py): 1e-4 for fp32 paths, 2e-2 for bf16 inputs with
fp32 accumulation, on max |g - r| / (|r| + rms(r)).
"""
import numpy as np
import pytest

import sfb_synth as S
from parity import TOL_BF16, TOL_F32, dml_follow_kink, max_rel, mlr_u_check, rel_err
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


def dev_bf16(a):
    return dev(S.bf16_bits(a)).view(torch.bfloat16)


def host(t):
    torch.cuda.synchronize()
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


# ---------------------------------------------------------------------------
# sfb_apply, fp32
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("N,J,D", [
    (32, 64, 128),          # smallest workload
    (2048, 1000, 2048),     # local + 7 peers; J not a multiple of any tile
    (7, 37, 50),            # nothing aligned: scalar load path
    (300, 129, 260),        # ragged tails in every dimension
    (33, 4, 2052),
    (65, 2052, 4),
])
def test_apply_f32_reconstruction_and_update(ctx, oracle, N, J, D):
    print("apply_f32", N, J, D, flush=True)
    g = np.random.default_rng(N * 7 + J)
    U = g.standard_normal((N, J), dtype=np.float32)
    V = g.standard_normal((N, D), dtype=np.float32)
    W0 = S.normal_matrix(J, D, 0.01, seed=5)
    # W = 0: pure reconstruction, -eta U^T V
    Wz = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    ctx.sfb_apply(Wz, dev(U), dev(V), 0.5)
    ref = oracle.apply(np.zeros((J, D)), U, V, 0.5)
    assert rel_err(host(Wz), ref) <= TOL_F32
    # W = W0, negative eta
    W = dev(W0)
    ctx.sfb_apply(W, dev(U), dev(V), -0.01)
    ref = oracle.apply(W0, U, V, -0.01)
    assert rel_err(host(W), ref) <= TOL_F32
    assert rel_err(host(W) - W0, ref - W0) <= TOL_F32


def test_apply_edge_cases(ctx, sfb, oracle):
    J, D = 40, 24
    W0 = S.normal_matrix(J, D, 0.01, seed=6)
    W = dev(W0)
    U = torch.zeros((0, J), dtype=torch.float32, device="cuda:0")
    V = torch.zeros((0, D), dtype=torch.float32, device="cuda:0")
    ctx.sfb_apply(W, U, V, 0.1)                       # N = 0: no-op
    np.testing.assert_array_equal(host(W), W0)
    # blocks applied one by one == concatenated (peer by peer), any order
    g = np.random.default_rng(3)
    Uh = g.standard_normal((48, J), dtype=np.float32); Vh = g.standard_normal((48, D), dtype=np.float32)
    Wa = dev(W0); ctx.sfb_apply(Wa, dev(Uh), dev(Vh), 0.01)
    Wb = dev(W0)
    for s in (slice(32, 48), slice(0, 32)):
        ctx.sfb_apply(Wb, dev(Uh[s]), dev(Vh[s]), 0.01)
    assert rel_err(host(Wb) - W0, host(Wa) - W0) <= TOL_F32
    # bit-reproducible
    Wc = dev(W0); ctx.sfb_apply(Wc, dev(Uh), dev(Vh), 0.01)
    np.testing.assert_array_equal(host(Wa), host(Wc))
    # argument errors come back as codes
    flat = torch.zeros(J * D + 1, dtype=torch.float32, device="cuda:0")
    with pytest.raises(sfb.SfbError) as e:
        ctx.sfb_apply(flat[1:].view(J, D), dev(Uh), dev(Vh), 0.1)      # W not 16-byte aligned
    assert e.value.code == sfb.SFB_EINVAL


# ---------------------------------------------------------------------------
# MLR, fp32
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("J,D,B", [(64, 128, 32), (1000, 2048, 256), (37, 50, 5), (513, 260, 130)])
def test_mlr_sf_f32(ctx, sfb, oracle, J, D, B):
    print("mlr_sf_f32", J, D, B, flush=True)
    W0 = S.normal_matrix(J, D, 0.05, seed=1)
    X, y = S.mlr_batch(J, D, B, seed=1)
    U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")
    ctx.sfb_compute_sf(sfb.SFB_MLR, dev(W0), dev(X), Y=dev(y), U=U, V=V)
    Uo, Vo = oracle.mlr_sf(W0, X, y)
    assert rel_err(host(U), Uo) <= TOL_F32
    mlr_u_check(host(U), Uo, y, TOL_F32)
    np.testing.assert_array_equal(host(V), X)
    assert np.max(np.abs(host(U).sum(axis=1))) < 1e-5


def test_mlr_large_logits_and_empty_batch(ctx, sfb, oracle):
    J, D, B = 96, 64, 16
    W0 = S.normal_matrix(J, D, 8.0, seed=2)            # logits of order +-60
    X, y = S.mlr_batch(J, D, B, seed=2)
    U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    ctx.sfb_compute_sf(sfb.SFB_MLR, dev(W0), dev(X), Y=dev(y), U=U)
    Uo, _ = oracle.mlr_sf(W0, X, y)
    assert np.all(np.isfinite(host(U)))
    assert rel_err(host(U), Uo) <= TOL_F32
    U0 = torch.empty((0, J), dtype=torch.float32, device="cuda:0")
    ctx.sfb_compute_sf(sfb.SFB_MLR, dev(W0), dev(X[:0]), Y=dev(y[:0]), U=U0)   # B = 0


def test_mlr_small_trajectory(ctx, sfb, oracle):
    c = S.CONFIGS["mlr_small"]
    J, D, B, eta = c["J"], c["D"], c["B"], c["eta"]
    W0 = S.normal_matrix(J, D, c["sigma"], seed=0)
    W = dev(W0); Wo = W0.astype(np.float64)
    U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    for step in range(c["steps"]):
        X, y = S.mlr_batch(J, D, B, seed=0, step=step)
        Xd = dev(X)
        ctx.sfb_compute_sf(sfb.SFB_MLR, W, Xd, Y=dev(y), U=U)
        ctx.sfb_apply(W, U, Xd, eta)
        Uo, Vo = oracle.mlr_sf(Wo, X, y)
        assert rel_err(host(U), Uo) <= TOL_F32
        mlr_u_check(host(U), Uo, y, TOL_F32)
        Wo = oracle.apply(Wo, Uo, Vo, eta)
    _trajectory_check(host(W), Wo, W0, c["steps"], TOL_F32)


def test_mlr_peers_trajectory(ctx, sfb, oracle):
    """Local batch plus 7 simulated peers' SF blocks, 2048 rank-1 terms a step."""
    c = S.CONFIGS["mlr_peers"]
    J, D, B, eta, P = c["J"], c["D"], c["B"], c["eta"], c["peers"]
    steps = c["steps"]                                   # all 20
    W0 = S.normal_matrix(J, D, c["sigma"], seed=0)
    W = dev(W0); Wo = W0.astype(np.float64)
    N = B * (P + 1)
    Uall = torch.empty((N, J), dtype=torch.float32, device="cuda:0")
    Vall = torch.empty((N, D), dtype=torch.float32, device="cuda:0")
    for step in range(steps):
        print("peers step", step, flush=True)
        X, y = S.mlr_batch(J, D, B, seed=0, step=step)
        peers = [S.mlr_peer_sf(J, D, B, seed=0, step=step, peer=p) for p in range(P)]
        for p, (Up, Vp) in enumerate(peers):
            Uall[B * (p + 1):B * (p + 2)] = dev(Up)
            Vall[B * (p + 1):B * (p + 2)] = dev(Vp)
        ctx.sfb_compute_sf(sfb.SFB_MLR, W, dev(X), Y=dev(y), U=Uall[:B], V=Vall[:B])
        ctx.sfb_apply(W, Uall, Vall, eta)
        Uo, Vo = oracle.mlr_sf(Wo, X, y)
        assert rel_err(host(Uall[:B]), Uo) <= TOL_F32
        mlr_u_check(host(Uall[:B]), Uo, y, TOL_F32)
        Ucat = np.concatenate([Uo] + [u for u, _ in peers]); Vcat = np.concatenate([Vo] + [v for _, v in peers])
        Wo = oracle.apply(Wo, Ucat, Vcat, eta)
    _trajectory_check(host(W), Wo, W0, steps, TOL_F32)


# ---------------------------------------------------------------------------
# MLR, bf16 inputs / fp32 W and accumulate
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("J,D,B", [(520, 328, 200), (1000, 2056, 257), (8, 8, 1), (264, 10000, 130),
                                   (40008, 264, 300),    # 314 tiles, more than one per persistent workgroup
                                   # rows long enough for the softmax that reads the logits once, several
                                   # workgroups per row: 2 per row with a ragged last tile; 4 per row, fewer rows
                                   # than clusters; 8 per row, rows in more than one round
                                   (70008, 136, 300), (160000, 72, 40), (170000, 72, 70)])
def test_mlr_sf_bf16(ctx, sfb, oracle, J, D, B):
    print("mlr_sf_bf16", J, D, B, flush=True)
    W0 = S.normal_matrix(J, D, 0.02 if J < 65536 else 0.2, seed=3)
    X, y = S.mlr_batch(J, D, B, seed=3, zero_frac=0.9, bf16=True)
    if J >= 65536:
        y[:4] = [0, J - 1, 255, 256]                  # labels at the ends of the row and of a tile
    U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
    ctx.sfb_compute_sf(sfb.SFB_MLR, dev(W0), dev_bf16(X), Y=dev(y), U=U)
    Uo, _ = oracle.mlr_sf(W0, X, y)
    got = host(U).astype(np.float64)
    assert rel_err(got, Uo) <= TOL_BF16
    print("  err", rel_err(got, Uo), max_rel(got, Uo))
    # The tolerance above is bf16's and its scale the label entry's: the probabilities are checked against
    # their own rms, each row's least-squares factor against 1, the label entry on its own.
    print("  masked err", mlr_u_check(got, Uo, y, TOL_BF16, factor_tol=2e-3 if J > 8 else None, label_tol=1e-2))


def test_mlr_softmax_partners_that_do_not_answer(sfb, oracle):
    """Long rows are shared by several workgroups that exchange one pair per row; a workgroup whose partner
    does not publish in time computes the partner's pair itself.  With a wait of zero polls every workgroup does
    so (whether or not the pair arrives meanwhile), and the factors are those of the ordinary run to rounding; two
    contexts whose kernels share the chip (neither set of workgroups is on it as a whole) finish with the same."""
    J, D, B = 170000, 72, 70
    W0 = S.normal_matrix(J, D, 0.2, seed=8)
    X, y = S.mlr_batch(J, D, B, seed=8, zero_frac=0.9, bf16=True)
    Uo, _ = oracle.mlr_sf(W0, X, y)
    Wd, Xd, yd = dev(W0), dev_bf16(X), dev(y)
    ca, cb = sfb.Context(0), sfb.Context(0)
    ca.sfb_shadow_attach(Wd); cb.sfb_shadow_attach(Wd)          # (each context keeps its own working copy)
    U0 = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
    ca.sfb_compute_sf(sfb.SFB_MLR, Wd, Xd, Y=yd, U=U0)
    torch.cuda.synchronize()
    assert rel_err(host(U0), Uo) <= TOL_BF16
    mlr_u_check(host(U0), Uo, y, TOL_BF16, label_tol=1e-2)
    before = ca.sfb_wait_fallbacks()
    ca.sfb_set_wait_limit(0)
    print("  zero polls", flush=True)
    U1 = torch.empty_like(U0)
    ca.sfb_compute_sf(sfb.SFB_MLR, Wd, Xd, Y=yd, U=U1)
    torch.cuda.synchronize()
    ca.sfb_set_wait_limit(-1)
    counted = ca.sfb_wait_fallbacks() - before
    print("  pairs computed by the waiting workgroup itself:", counted, flush=True)
    assert counted >= 8 * 7                         # 8 workgroups a row, each does its 7 partners' parts (at least in its first row)
    assert rel_err(host(U1), Uo) <= TOL_BF16
    mlr_u_check(host(U1), Uo, y, TOL_BF16, label_tol=1e-2)
    same = float((U1 == U0).float().mean())
    print("  identical entries with and without waiting: %.6f" % same, flush=True)
    assert same > 0.99 and rel_err(host(U1), host(U0)) <= 1e-2
    print("  two contexts at once", flush=True)
    Ua, Ub = torch.empty_like(U0), torch.empty_like(U0)
    for _ in range(3):
        ca.sfb_compute_sf(sfb.SFB_MLR, Wd, Xd, Y=yd, U=Ua)
        cb.sfb_compute_sf(sfb.SFB_MLR, Wd, Xd, Y=yd, U=Ub)
    torch.cuda.synchronize()
    for U in (Ua, Ub):
        assert rel_err(host(U), Uo) <= TOL_BF16
        mlr_u_check(host(U), Uo, y, TOL_BF16, label_tol=1e-2)
        assert float((U == U0).float().mean()) > 0.99
    ca.close(); cb.close()


@pytest.mark.parametrize("N,J,D", [(1024, 520, 328), (100, 1000, 2056), (1, 8, 8), (77, 264, 136), (130, 128, 128),
                                   (100, 4104, 4104),     # 289 tiles: several per persistent workgroup, ragged both ways
                                   (2100, 264, 520)])     # k longer than the headline's, not a multiple of 64
def test_apply_bf16(ctx, sfb, oracle, N, J, D):
    print("apply_bf16", N, J, D, flush=True)
    U, V = S.mlr_peer_sf(J, D, N, seed=4, step=0, peer=0, bf16=True)
    Wz = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    ctx.sfb_apply(Wz, dev_bf16(U), dev_bf16(V), 1.0)
    ref = oracle.apply(np.zeros((J, D)), U, V, 1.0)
    assert rel_err(host(Wz), ref) <= TOL_F32            # bf16 products are exact in fp32: only the sum order differs
    W0 = S.normal_matrix(J, D, 0.01, seed=4)
    W = dev(W0)
    ctx.sfb_apply(W, dev_bf16(U), dev_bf16(V), 0.001)
    ref = oracle.apply(W0, U, V, 0.001)
    _trajectory_check(host(W), ref, W0, 1, TOL_F32)


def test_apply_bf16_local_plus_seven_peer_blocks(ctx, sfb, oracle):
    """One worker's share of a broadcast step with eight workers (Section 3: every worker applies the factor
    sets of all workers): eight blocks of 1024 + a ragged 37 rows in one call (k = 8229, 129 slices) against the
    oracle, and the same blocks applied one call each (the sum is the same up to the order of additions)."""
    J, D, P = 520, 328, 8
    blocks = [S.mlr_peer_sf(J, D, 1024 if q < P else 37, seed=5, step=0, peer=q, bf16=True) for q in range(P + 1)]
    U = np.concatenate([b[0] for b in blocks]); V = np.concatenate([b[1] for b in blocks])
    W0 = S.normal_matrix(J, D, 0.01, seed=5)
    W = dev(W0)
    ctx.sfb_apply(W, dev_bf16(U), dev_bf16(V), 0.001)
    ref = oracle.apply(W0, U, V, 0.001)
    _trajectory_check(host(W), ref, W0, 1, TOL_F32)
    W2 = dev(W0)
    for Ub, Vb in blocks:
        ctx.sfb_apply(W2, dev_bf16(Ub), dev_bf16(Vb), 0.001)
    _trajectory_check(host(W2), ref, W0, len(blocks), TOL_F32)
    # on the two planes as well (the benchmark's layout)
    c2 = sfb.Context(0)
    W3 = dev(W0)
    c2.sfb_split_attach(W3)
    c2.sfb_apply(W3, dev_bf16(U), dev_bf16(V), 0.001)
    c2.sfb_split_export(W3)
    torch.cuda.synchronize()
    assert torch.equal(W3, W)
    c2.close()


def test_bf16_shadow_stays_current(sfb, oracle):
    """With a bf16 working copy of W attached, SFs after several applies (and a prox) equal those of a
    context that converts W afresh on every call, bit for bit."""
    J, D, B, eta = 520, 328, 200, 0.05
    W0 = S.normal_matrix(J, D, 0.05, seed=21)
    ca, cb = sfb.Context(0), sfb.Context(0)
    Wa, Wb = dev(W0), dev(W0)
    ca.sfb_shadow_attach(Wa)
    Ua = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0"); Ub = torch.empty_like(Ua)
    for step in range(3):
        X, y = S.mlr_batch(J, D, B, seed=21, step=step, zero_frac=0.5, bf16=True)
        Xd, yd = dev_bf16(X), dev(y)
        ca.sfb_compute_sf(sfb.SFB_MLR, Wa, Xd, Y=yd, U=Ua)
        cb.sfb_compute_sf(sfb.SFB_MLR, Wb, Xd, Y=yd, U=Ub)
        assert torch.equal(Ua, Ub), step
        if step == 2:
            Uo, _ = oracle.mlr_sf(host(Wb), X, y)
            assert rel_err(host(Ua), Uo) <= TOL_BF16
            mlr_u_check(host(Ua), Uo, y, TOL_BF16, label_tol=1e-2)
        before = Wb.bfloat16()
        step_eta = eta if step != 1 else eta * 1e-4          # the small one leaves most bf16 values as they are
        ca.sfb_apply(Wa, Ua, Xd, step_eta); cb.sfb_apply(Wb, Ub, Xd, step_eta)
        assert torch.equal(Wa, Wb)
        # the copy is rewritten four columns at a time, and only where its bits change: both cases must occur
        moved = (Wb.bfloat16() != before).view(J, D // 4, 4).any(dim=2).float().mean().item()
        print("  groups of four whose bf16 value changed: %.3f" % moved, flush=True)
        assert moved > 0.0 and (step != 1 or moved < 0.9)
        if step == 1:
            ca.sfb_prox_rows(Wa, sfb.SFB_PROX_PROJECT); cb.sfb_prox_rows(Wb, sfb.SFB_PROX_PROJECT)
    # a caller-side change of W must be followed by a refresh
    Wa.mul_(0.5); Wb.mul_(0.5)
    ca.sfb_shadow_attach(Wa)
    ca.sfb_compute_sf(sfb.SFB_MLR, Wa, Xd, Y=yd, U=Ua)
    cb.sfb_compute_sf(sfb.SFB_MLR, Wb, Xd, Y=yd, U=Ub)
    assert torch.equal(Ua, Ub)
    ca.close(); cb.close()


def test_bf16_rejects_unaligned_shapes(ctx, sfb):
    W = torch.zeros((12, 16), dtype=torch.float32, device="cuda:0")       # J % 8 != 0
    U = torch.zeros((4, 12), dtype=torch.bfloat16, device="cuda:0")
    V = torch.zeros((4, 16), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(sfb.SfbError) as e:
        ctx.sfb_apply(W, U, V, 0.1)
    assert e.value.code == sfb.SFB_EINVAL


# ---------------------------------------------------------------------------
# Signed low-rank updates (one coefficient per factor pair)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("N,J,D", [(2, 200, 136), (333, 264, 520), (1, 8, 8), (600, 1000, 264)])
def test_apply_signed_f32(ctx, sfb, oracle, N, J, D):
    print("apply_signed_f32", N, J, D, flush=True)
    g = np.random.default_rng([55, N])
    U = g.standard_normal((N, J), dtype=np.float32)
    V = g.standard_normal((N, D), dtype=np.float32)
    c = g.standard_normal(N).astype(np.float32)
    W0 = S.normal_matrix(J, D, 1.0, seed=5)
    W = dev(W0)
    ctx.sfb_apply_signed(W, dev(U), dev(V), dev(c), 0.05)
    Wo = oracle.apply_signed(W0, U, V, c, 0.05)
    assert rel_err(host(W) - W0, Wo - W0) <= TOL_F32


@pytest.mark.parametrize("N,J,D,unit", [(2, 264, 136, True), (300, 520, 328, True), (300, 520, 328, False),
                                        (1024, 264, 4104, False)])
def test_apply_signed_bf16(ctx, sfb, oracle, N, J, D, unit):
    print("apply_signed_bf16", N, J, D, unit, flush=True)
    U, V = S.mlr_peer_sf(J, D, N, seed=6, step=0, peer=0, bf16=True)
    g = np.random.default_rng([56, N])
    c = (g.integers(0, 2, N) * 2 - 1).astype(np.float32) if unit else g.standard_normal(N).astype(np.float32)
    W0 = S.normal_matrix(J, D, 1.0, seed=6)
    W = dev(W0)
    ctx.sfb_apply_signed(W, dev_bf16(U), dev_bf16(V), dev(c), 0.05)
    Wo = oracle.apply_signed(W0, U, V, c, 0.05)
    # +-1 coefficients are exact in bf16: only the summation order differs; otherwise c * v is rounded to bf16
    assert rel_err(host(W) - W0, Wo - W0) <= (TOL_F32 if unit else TOL_BF16)


def test_apply_signed_rejects_bad_arguments(ctx, sfb):
    W = torch.zeros((16, 16), dtype=torch.float32, device="cuda:0")
    U = torch.zeros((4, 16), dtype=torch.float32, device="cuda:0")
    L = sfb.lib()
    import ctypes
    rc = L.sfb_apply_signed(ctx._h, W.data_ptr(), 16, 16, U.data_ptr(), U.data_ptr(), None, 4, sfb.SFB_F32,
                            ctypes.c_float(0.1))
    assert rc == sfb.SFB_EINVAL                     # no coefficients


# ---------------------------------------------------------------------------
# DML
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("K,D,B,sigma", [
    (1024, 4096, 512, 0.01),                       # the workload as stated: every hinge term inactive
    (1024, 4096, 512, (2 * 1024 * 4096) ** -0.5),  # E||W(x-y)||^2 ~ 1: about half the hinge terms active
    (33, 70, 9, 0.05),
])
def test_dml_sf(ctx, sfb, oracle, K, D, B, sigma):
    print("dml", K, D, B, sigma, flush=True)
    W0 = S.normal_matrix(K, D, sigma, seed=7)
    X, Y, sim = S.dml_batch(D, B, seed=7)
    U = torch.empty((B, K), dtype=torch.float32, device="cuda:0")
    V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")
    na = torch.full((1,), -5, dtype=torch.int32, device="cuda:0")
    ctx.sfb_compute_sf(sfb.SFB_DML, dev(W0), dev(X), Y=dev(Y), sim=dev(sim), U=U, V=V, n_active=na, margin=1.0)
    Uo, Vo, no = oracle.dml_sf(W0, X, Y, sim, margin=1.0)
    d = np.sum(((X.astype(np.float64) - Y) @ W0.T.astype(np.float64)) ** 2, axis=1)
    assert np.min(np.abs(d[sim < 0] - 1.0)) > 1e-5        # no pair within fp32 rounding of the kink: the decision is unique
    assert int(host(na)[0]) == no
    print("  n_active", no, "of", B)
    np.testing.assert_array_equal(host(V), (X - Y).astype(np.float32))
    assert rel_err(host(U), Uo) <= TOL_F32
    np.testing.assert_array_equal(np.all(host(U) == 0, axis=1), np.all(Uo == 0, axis=1))


def test_dml_hinge_ties_by_hand(ctx, sfb, oracle):
    K, D = 8, 8
    W0 = np.eye(K, D, dtype=np.float32)
    X = np.zeros((4, D), dtype=np.float32); Y = np.zeros((4, D), dtype=np.float32)
    X[0, 0] = 1.0                    # d = 1 exactly: tie -> inactive
    X[1, 0] = 0.5; X[1, 1] = 0.5     # d = 0.5: active
    X[2, 0] = 1.0; X[2, 3] = 0.25    # d = 1.0625: inactive
    X[3, 2] = 3.0                    # similar pair, d = 9
    sim = np.array([-1, -1, -1, 1], dtype=np.int8)
    U = torch.empty((4, K), dtype=torch.float32, device="cuda:0")
    V = torch.empty((4, D), dtype=torch.float32, device="cuda:0")
    na = torch.zeros((1,), dtype=torch.int32, device="cuda:0")
    ctx.sfb_compute_sf(sfb.SFB_DML, dev(W0), dev(X), Y=dev(Y), sim=dev(sim), U=U, V=V, n_active=na)
    Uo, Vo, no = oracle.dml_sf(W0, X, Y, sim)
    np.testing.assert_array_equal(host(U), Uo.astype(np.float32))
    assert int(host(na)[0]) == no == 2


@pytest.mark.parametrize("variant", ["stated", "half_active"])
def test_dml_trajectory(ctx, sfb, oracle, variant):
    """The metric-learning workload at its stated size and step count: 10 steps of SF computation +
    application, a fresh batch of pairs per step, the oracle's W kept in fp64.  As stated (W ~ N(0, 0.01^2))
    every hinge term is inactive; the second variant starts where about half of them are active."""
    c = S.CONFIGS["dml"]
    K, D, B, eta, steps = c["K"], c["D"], c["B"], c["eta"], c["steps"]
    sigma = c["sigma"] if variant == "stated" else (2.0 * K * D) ** -0.5
    W0 = S.normal_matrix(K, D, sigma, seed=0)
    W = dev(W0); Wo = W0.astype(np.float64)
    U = torch.empty((B, K), dtype=torch.float32, device="cuda:0")
    V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")
    na = torch.zeros((1,), dtype=torch.int32, device="cuda:0")
    n_near = 0
    for step in range(steps):
        X, Y, sim = S.dml_batch(D, B, seed=0, step=step)
        ctx.sfb_compute_sf(sfb.SFB_DML, W, dev(X), Y=dev(Y), sim=dev(sim), U=U, V=V, n_active=na, margin=c["margin"])
        ctx.sfb_apply(W, U, V, eta)
        Uo, Vo, no = oracle.dml_sf(Wo, X, Y, sim, margin=c["margin"])
        Ug = host(U)
        Uo, no, near = dml_follow_kink(oracle, Uo, no, Ug, Wo, X, Y, sim, c["margin"], 1e-4)
        n_near += near
        print("  dml step", step, "active", no, "pairs at the kink", near, flush=True)
        assert int(host(na)[0]) == no
        assert rel_err(Ug, Uo) <= TOL_F32
        Wo = oracle.apply(Wo, Uo, Vo, eta)
    _trajectory_check(host(W), Wo, W0, steps, TOL_F32)


# ---------------------------------------------------------------------------
# sparse coding
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("J,D,B", [(256, 96, 40), (70, 33, 9), (1024, 512, 192)])
def test_sc_sf(ctx, sfb, oracle, J, D, B):
    print("sc", J, D, B, flush=True)
    W0 = S.sc_dictionary(J, D, seed=8)
    X = S.sc_batch(D, B, seed=8)
    U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")
    ctx.sfb_compute_sf(sfb.SFB_SC, dev(W0), dev(X), U=U, V=V, lam=0.1, ista_iters=20, power_iters=10)
    Uo, Vo, L = oracle.sc_sf(W0, X, lam=0.1, ista_iters=20, power_iters=10)
    print("  L", L, "nnz frac", np.mean(Uo != 0), "errs", rel_err(host(U), Uo), rel_err(host(V), Vo))
    assert rel_err(host(U), Uo) <= TOL_F32
    assert rel_err(host(V), Vo) <= TOL_F32


def test_sc_full_step_with_prox(ctx, sfb, oracle):
    """The sparse-coding workload at full size: SFs, W += eta U^T V, row projection."""
    c = S.CONFIGS["sc"]
    J, D, B, eta = c["J"], c["D"], c["B"], c["eta"]
    W0 = S.sc_dictionary(J, D, seed=0)
    X = S.sc_batch(D, B, seed=0)
    W = dev(W0)
    U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")
    print("sc full: gpu", flush=True)
    ctx.sfb_compute_sf(sfb.SFB_SC, W, dev(X), U=U, V=V, lam=c["lam"], ista_iters=c["ista_iters"],
                       power_iters=c["power_iters"])
    ctx.sfb_apply(W, U, V, -eta)
    Wn = W.clone()
    ctx.sfb_prox_rows(W, sfb.SFB_PROX_PROJECT)
    ctx.sfb_prox_rows(Wn, sfb.SFB_PROX_NORMALIZE)
    print("sc full: oracle", flush=True)
    Uo, Vo, L = oracle.sc_sf(W0, X, lam=c["lam"], ista_iters=c["ista_iters"], power_iters=c["power_iters"])
    assert rel_err(host(U), Uo) <= TOL_F32
    assert rel_err(host(V), Vo) <= TOL_F32
    W1 = oracle.apply(W0, Uo, Vo, -eta)
    for Wg, mode in ((W, oracle.PROX_PROJECT), (Wn, oracle.PROX_NORMALIZE)):
        ref = oracle.prox_rows(W1, mode)
        assert rel_err(host(Wg), ref) <= TOL_F32
        assert np.max(np.linalg.norm(host(Wg).astype(np.float64), axis=1)) <= 1 + 1e-6


@pytest.mark.timeout(600)
def test_sc_trajectory(ctx, sfb, oracle):
    """The sparse-coding workload at its stated dictionary size and step count: 5 steps of code solve,
    W += eta U^T V and row projection, a fresh batch per step, against the oracle's fp64 trajectory.  The batch
    is the stated 512 samples (the oracle's un-blocked loops need a quarter of a minute per step on the GPU machine's
    host cores)."""
    c = S.CONFIGS["sc"]
    J, D, eta, steps = c["J"], c["D"], c["eta"], c["steps"]
    B = c["B"]
    W0 = S.sc_dictionary(J, D, seed=0)
    W = dev(W0); Wo = W0.astype(np.float64)
    U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")
    for step in range(steps):
        X = S.sc_batch(D, B, seed=0, step=step)
        ctx.sfb_compute_sf(sfb.SFB_SC, W, dev(X), U=U, V=V, lam=c["lam"], ista_iters=c["ista_iters"],
                           power_iters=c["power_iters"])
        ctx.sfb_apply(W, U, V, -eta)
        ctx.sfb_prox_rows(W, sfb.SFB_PROX_PROJECT)
        Uo, Vo, L = oracle.sc_sf(Wo, X, lam=c["lam"], ista_iters=c["ista_iters"], power_iters=c["power_iters"])
        print("  sc step", step, "L", L, "errs", rel_err(host(U), Uo), rel_err(host(V), Vo), flush=True)
        assert rel_err(host(U), Uo) <= TOL_F32
        assert rel_err(host(V), Vo) <= TOL_F32
        Wo = oracle.prox_rows(oracle.apply(Wo, Uo, Vo, -eta), oracle.PROX_PROJECT)
    _trajectory_check(host(W), Wo, W0, steps, TOL_F32)
    assert np.max(np.linalg.norm(host(W).astype(np.float64), axis=1)) <= 1 + 1e-6


def test_prox_rows(ctx, sfb, oracle):
    g = np.random.default_rng(9)
    W0 = g.standard_normal((67, 130)).astype(np.float32) * 0.12
    W0[3] = 0.0
    W0[5] *= 0.01
    for mode_g, mode_o in ((sfb.SFB_PROX_PROJECT, oracle.PROX_PROJECT), (sfb.SFB_PROX_NORMALIZE, oracle.PROX_NORMALIZE)):
        W = dev(W0)
        ctx.sfb_prox_rows(W, mode_g)
        ref = oracle.prox_rows(W0, mode_o)
        assert rel_err(host(W), ref) <= TOL_F32
        if mode_g == sfb.SFB_PROX_PROJECT:
            inside = np.linalg.norm(W0.astype(np.float64), axis=1) <= 1.0
            assert inside.any() and (~inside).any()
            np.testing.assert_array_equal(host(W)[inside], W0[inside])     # untouched rows stay bit-identical
            W2 = W.clone(); ctx.sfb_prox_rows(W2, mode_g)
            assert rel_err(host(W2), host(W)) <= 1e-6                     # idempotent


def test_workspace_too_small_is_reported(sfb):
    c = sfb.Context(0)
    J, D, B = 64, 32, 16
    W = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    X = torch.zeros((B, D), dtype=torch.float32, device="cuda:0")
    y = torch.zeros((B,), dtype=torch.int32, device="cuda:0")
    U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
    b = sfb.sfb_batch()
    b.X = X.data_ptr(); b.Y = y.data_ptr(); b.B = B; b.in_dtype = 0; b.sf_dtype = 0
    import ctypes
    rc = sfb.lib().sfb_compute_sf(c._h, sfb.SFB_MLR, W.data_ptr(), J, D, ctypes.byref(b), U.data_ptr(), None, None)
    assert rc == sfb.SFB_ENOWS
    c.close()
