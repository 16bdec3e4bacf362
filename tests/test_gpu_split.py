"""GPU tests of the split storage of W (two 16-bit planes, sfb_split_*): exact
round trip, sfb_apply on the planes bit-identical to sfb_apply on the fp32 array,
the forward contraction on the high plane against the oracle, and the calls that
must refuse a matrix whose fp32 array is stale.
"""
import numpy as np
import pytest

import sfb_synth as S
from parity import TOL_BF16, TOL_F32, mlr_u_check, rel_err, trajectory_check

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


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


def test_split_round_trip_is_exact(sfb):
    J, D = 264, 328
    g = np.random.default_rng(31)
    bits = g.integers(0, 2 ** 32, size=(J, D), dtype=np.uint64).astype(np.uint32)      # every kind of bit pattern
    special = np.array([0x00000000, 0x80000000, 0x00008000, 0x00007fff, 0x0000ffff, 0x3f808000, 0x3f807fff, 0x3f80ffff,
                        0xbf808000, 0x7f7fffff, 0xff7fffff, 0x7f800000, 0xff800000, 0x7fc00001, 0xffffffff, 0x00000001],
                       dtype=np.uint32)
    bits[0, :16] = special
    W = dev(bits.view(np.int32)).view(torch.float32)
    before = W.view(torch.int32).clone()
    c = sfb.Context(0)
    c.sfb_split_attach(W)
    W.zero_()                                        # the planes, not the fp32 array, hold the parameters now
    c.sfb_split_export(W)
    torch.cuda.synchronize()
    assert torch.equal(W.view(torch.int32), before)
    c.sfb_split_detach()
    c.close()


@pytest.mark.parametrize("N,J,D,kind", [
    (1024, 520, 328, "plain"),
    (100, 4104, 4104, "plain"),      # 289 tiles, ragged both ways
    (2100, 264, 520, "plain"),
    (1, 8, 8, "plain"),
    (333, 264, 520, "signed"),
    (700, 1000, 2056, "csr"),
    (600, 520, 328, "small"),        # steps so small that most groups of four keep their high halves
])
def test_apply_on_planes_gives_the_bits_of_apply_on_fp32(sfb, oracle, N, J, D, kind):
    print("split apply", N, J, D, kind, flush=True)
    U, V = S.mlr_peer_sf(J, D, N, seed=12, step=0, peer=0, bf16=True)
    if kind == "csr":
        V, _ = S.mlr_batch(J, D, N, seed=12, step=1, zero_frac=0.9, bf16=True)
    W0 = S.normal_matrix(J, D, 0.01, seed=12)
    Wa, Wb = dev(W0), dev(W0)
    ca, cb = sfb.Context(0), sfb.Context(0)
    cb.sfb_split_attach(Wb)
    coef = dev(np.where(np.arange(N) % 2 == 0, 1.0, -1.0).astype(np.float32))
    Ud, Vd = dev_bf16(U), dev_bf16(V)
    csr = None
    if kind == "csr":
        ip, ix, vals = S.csr_from_dense(V)
        csr = (dev(ip), dev(ix), dev(S.bf16_bits(vals)).view(torch.bfloat16))
    etas = (0.001, -0.0005, 0.002) if kind != "small" else (2e-6, -1e-6, 4e-6)
    for step, eta in enumerate(etas):                            # several updates on top of each other
        for c, W in ((ca, Wa), (cb, Wb)):
            if kind in ("plain", "small"):
                c.sfb_apply(W, Ud, Vd, eta)
            elif kind == "signed":
                c.sfb_apply_signed(W, Ud, Vd, coef, eta)
            else:
                c.sfb_apply_csr(W, Ud, csr[0], csr[1], csr[2], eta)
    torch.cuda.synchronize()
    assert torch.equal(Wb, dev(W0))                  # the fp32 array of the split matrix was not touched
    cb.sfb_split_export(Wb)
    torch.cuda.synchronize()
    assert torch.equal(Wa, Wb)
    if J * D > 10000:
        # the high plane is rewritten four columns at a time, and only where it changes: the case must hold both kinds
        hi = lambda W: (W.view(torch.int32).to(torch.int64) + 0x8000) >> 16
        moved = (hi(Wb) != hi(dev(W0))).view(J, D // 4, 4).any(dim=2).float().mean().item()
        print("  groups of four whose high half changed: %.3f" % moved, flush=True)
        assert moved > 0.0 and (kind != "small" or moved < 0.5)
    if kind == "plain" and J * D * N < 2e9:
        ref = W0.astype(np.float64)
        for eta in etas:
            ref = oracle.apply(ref, U, V, eta)
        trajectory_check(host(Wb), ref, W0, len(etas), TOL_F32)
    ca.close(); cb.close()


@pytest.mark.parametrize("J,D,B", [(520, 328, 200), (1000, 2056, 257), (40008, 264, 300)])
def test_forward_on_the_high_plane(sfb, oracle, J, D, B):
    print("split forward", J, D, B, flush=True)
    W0 = S.normal_matrix(J, D, 0.02, seed=13)
    X, y = S.mlr_batch(J, D, B, seed=13, zero_frac=0.9, bf16=True)
    ca, cb = sfb.Context(0), sfb.Context(0)
    Wa, Wb = dev(W0), dev(W0)
    ca.sfb_shadow_attach(Wa)
    cb.sfb_split_attach(Wb)
    Ua = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0"); Ub = torch.empty_like(Ua)
    ca.sfb_compute_sf(sfb.SFB_MLR, Wa, dev_bf16(X), Y=dev(y), U=Ua)
    cb.sfb_compute_sf(sfb.SFB_MLR, Wb, dev_bf16(X), Y=dev(y), U=Ub)
    Uo, _ = oracle.mlr_sf(W0, X, y)
    assert rel_err(host(Ub), Uo) <= TOL_BF16
    mlr_u_check(host(Ub), Uo, y, TOL_BF16, label_tol=1e-2)
    # the high plane differs from the round-to-nearest-even working copy only where the dropped half is an
    # exact tie: almost every factor is the same bf16 number
    same = float((Ua == Ub).float().mean())
    print("  identical entries: %.6f" % same, flush=True)
    assert same > 0.99 and rel_err(host(Ub), host(Ua)) <= 2e-2
    # CSR samples take the same route
    ip, ix, vals = S.csr_from_dense(X)
    Uc = torch.empty_like(Ub)
    cb.sfb_mlr_sf_csr(Wb, dev(ip), dev(ix), dev(S.bf16_bits(vals)).view(torch.bfloat16), dev(y), Uc)
    torch.cuda.synchronize()
    assert torch.equal(Uc, Ub)
    ca.close(); cb.close()


def test_split_training_steps_against_the_oracle(sfb, oracle):
    """Three whole steps (SF computation + application) on the planes, then export."""
    J, D, B, eta = 520, 328, 200, 0.05
    W0 = S.normal_matrix(J, D, 0.05, seed=14)
    c = sfb.Context(0)
    W = dev(W0)
    c.sfb_split_attach(W)
    Wo = W0.astype(np.float64)
    U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
    for step in range(3):
        X, y = S.mlr_batch(J, D, B, seed=14, step=step, zero_frac=0.5, bf16=True)
        Xd = dev_bf16(X)
        c.sfb_compute_sf(sfb.SFB_MLR, W, Xd, Y=dev(y), U=U)
        c.sfb_apply(W, U, Xd, eta)
        Uo, _ = oracle.mlr_sf(Wo, X, y)
        mlr_u_check(host(U), Uo, y, TOL_BF16, label_tol=1e-2)
        Wo = oracle.apply(Wo, Uo, X, eta)
    c.sfb_split_export(W)
    got = host(W)
    assert rel_err(got - W0, Wo - W0) <= TOL_BF16
    c.close()


def test_split_refuses_what_would_use_the_stale_array(sfb):
    J, D, B = 16, 24, 4
    W = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    c = sfb.Context(0)
    c.sfb_split_attach(W)
    Uf = torch.zeros((B, J), device="cuda:0"); Vf = torch.zeros((B, D), device="cuda:0")
    y = torch.zeros((B,), dtype=torch.int32, device="cuda:0")
    Xb = torch.zeros((B, D), dtype=torch.bfloat16, device="cuda:0")
    Ub = torch.zeros((B, 8), dtype=torch.bfloat16, device="cuda:0")
    for call in (lambda: c.sfb_apply(W, Uf, Vf, 0.1),
                 lambda: c.sfb_compute_sf(sfb.SFB_MLR, W[:8], Xb, Y=y, U=Ub),      # the attached pointer, another shape
                 lambda: c.sfb_apply(W[:8], Ub, Xb, 0.1),
                 lambda: c.sfb_prox_rows(W),
                 lambda: c.sfb_compute_sf(sfb.SFB_MLR, W, Vf, Y=y, U=Uf),
                 lambda: c.sfb_sdca_mlr_sf(W, Vf, torch.full((B, J), 1.0 / J, device="cuda:0"), 0.1, 10, 1.0, Uf),
                 lambda: c.sfb_dual_to_primal_l2(W, W, 0.1),
                 lambda: c.sfb_shadow_attach(W)):
        with pytest.raises(sfb.SfbError) as e:
            call()
        assert e.value.code == sfb.SFB_EINVAL
    other = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    c.sfb_apply(other, Uf, Vf, 0.1)                  # other matrices are unaffected
    c.sfb_split_detach()
    c.sfb_apply(W, Uf, Vf, 0.1)                      # and after detaching W is an ordinary fp32 matrix again
    with pytest.raises(sfb.SfbError):
        c.sfb_split_export(W)
    torch.cuda.synchronize()
    c.close()
