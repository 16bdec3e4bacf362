"""GPU parity of the CSR entry points (sparse samples / sparse second factors)
against the CPU oracle's loops over the stored non-zeros, and bit-equality with
the dense entry points on the same data.
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


@pytest.fixture(scope="module")
def ctx(sfb):
    c = sfb.Context(0)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def dev_vals(a, bf16):
    return dev(S.bf16_bits(a)).view(torch.bfloat16) if bf16 else dev(a.astype(np.float32))


def host(t):
    torch.cuda.synchronize()
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


def csr_dev(X, bf16):
    indptr, indices, values = S.csr_from_dense(X)
    return (indptr, indices, values), (dev(indptr), dev(indices), dev_vals(values, bf16))


@pytest.mark.parametrize("route", [1, 2])                  # 1: dense product on operands written from the CSR rows; 2: over the stored entries
@pytest.mark.parametrize("J,D,B,bf16,zero_frac", [
    (64, 128, 32, False, 0.9),
    (1000, 2048, 256, False, 0.9),
    (37, 50, 7, False, 0.5),        # nothing aligned
    (1000, 7000, 300, False, 0.99), # 1 % non-zeros; three column chunks; J not a multiple of the 32-class groups
    (520, 328, 200, True, 0.9),
    (264, 10000, 130, True, 0.9),   # the headline's feature count: four column chunks
    (40008, 264, 300, True, 0.97),  # several tiles per workgroup; some samples nearly empty
    (2056, 10000, 1100, True, 0.998),   # 0.2 % non-zeros; more samples than one group of 1024, last slice ragged
    (70008, 1000, 130, True, 0.99),     # 1 % non-zeros; rows long enough for the softmax that shares a row
])
def test_mlr_sf_csr(ctx, sfb, oracle, J, D, B, bf16, zero_frac, route):
    print("mlr_sf_csr", J, D, B, bf16, zero_frac, "route", route, flush=True)
    W0 = S.normal_matrix(J, D, 0.02 if zero_frac < 0.98 else 0.2, seed=5)
    X, y = S.mlr_batch(J, D, B, seed=5, zero_frac=zero_frac, bf16=bf16)
    X[B // 2] = 0.0                                            # one sample without any non-zero
    (indptr, indices, values), (ip, ix, vals) = csr_dev(X, bf16)
    dt = torch.bfloat16 if bf16 else torch.float32
    U = torch.empty((B, J), dtype=dt, device="cuda:0")
    assert ctx.sfb_csr_check(ip, ix, vals, D) == 0
    ctx.sfb_set_csr_route(route)
    try:
        ctx.sfb_profile_enable(True)
        ctx.sfb_profile_collect()
        ctx.sfb_mlr_sf_csr(dev(W0), ip, ix, vals, dev(y), U)
        ran = ctx.sfb_profile_collect()
    finally:
        ctx.sfb_profile_enable(False)
        ctx.sfb_set_csr_route(0)
    assert ("csr_forward_gather" in ran) == (route == 2), ran      # the route asked for is the one that ran
    Uo = oracle.mlr_sf_csr(W0, indptr, indices, values, y)
    err = rel_err(host(U), Uo)
    print("  err", err, flush=True)
    assert err <= (TOL_BF16 if bf16 else TOL_F32)
    if bf16:
        mlr_u_check(host(U), Uo, y, TOL_BF16, label_tol=1e-2)
    else:
        mlr_u_check(host(U), Uo, y, TOL_F32)
    Ud = torch.empty_like(U)
    ctx.sfb_compute_sf(sfb.SFB_MLR, dev(W0), dev_vals(X, bf16).reshape(B, D), Y=dev(y), U=Ud)
    if route == 1:
        # same kernels on the same operand values as the dense entry point: same bits
        assert torch.equal(U, Ud)
    else:
        # another summation order: the same numbers up to the rounding of the output type
        same = float((U == Ud).float().mean())
        print("  entries identical to the dense route's: %.4f" % same, flush=True)
        assert rel_err(host(U), host(Ud)) <= (TOL_BF16 if bf16 else TOL_F32)
        assert not bf16 or same > 0.9


def test_mlr_sf_csr_picks_its_route(ctx, sfb):
    """Left to itself, the call goes over the stored entries at a fraction of a per cent of non-zeros and through
    the dense product at ten per cent."""
    J, D, B = 4096, 4096, 512
    W = dev(S.normal_matrix(J, D, 0.02, seed=9))
    U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
    for zero_frac, want in ((0.998, True), (0.9, False)):
        X, y = S.mlr_batch(J, D, B, seed=9, zero_frac=zero_frac, bf16=True)
        _, (ip, ix, vals) = csr_dev(X, True)
        ctx.sfb_profile_enable(True)
        ctx.sfb_profile_collect()
        ctx.sfb_mlr_sf_csr(W, ip, ix, vals, dev(y), U)
        ran = ctx.sfb_profile_collect()
        ctx.sfb_profile_enable(False)
        assert ("csr_forward_gather" in ran) == want, (zero_frac, ran)


@pytest.mark.parametrize("N,J,D,bf16,zero_frac,signed", [
    (32, 64, 128, False, 0.9, False),
    (2048, 1000, 2048, False, 0.9, False),
    (7, 37, 50, False, 0.5, True),
    (1024, 520, 328, True, 0.9, False),
    (100, 4104, 4104, True, 0.99, False),   # 289 tiles; most columns untouched
    (2100, 264, 520, True, 0.9, True),
])
def test_apply_csr(ctx, sfb, oracle, N, J, D, bf16, zero_frac, signed):
    print("apply_csr", N, J, D, bf16, signed, flush=True)
    U, _ = S.mlr_peer_sf(J, D, N, seed=6, step=0, peer=0, bf16=bf16)
    V, _ = S.mlr_batch(J, D, N, seed=6, step=1, zero_frac=zero_frac, bf16=bf16)
    V[N // 3] = 0.0
    (indptr, indices, values), (ip, ix, vals) = csr_dev(V, bf16)
    coef = None
    coef_d = None
    if signed:
        coef = np.where(np.arange(N) % 3 == 0, -1.0, 1.0).astype(np.float32)
        coef_d = dev(coef)
    W0 = S.normal_matrix(J, D, 0.01, seed=6)
    W = dev(W0)
    eta = 0.001
    ctx.sfb_apply_csr(W, dev_vals(U, bf16), ip, ix, vals, eta, coef=coef_d)
    Ueff = U if coef is None else U * coef[:, None]            # exact for +-1
    ref = oracle.apply_csr(W0, Ueff, indptr, indices, values, eta)
    got = host(W)
    print("  update err", rel_err(got - W0, ref - W0), flush=True)
    trajectory_check(got, ref, W0, 1, TOL_F32)                  # the update itself, up to the rounding of the stored W
    assert rel_err(got, ref) <= TOL_F32
    # columns no factor touches keep their bits
    touched = np.zeros(D, bool)
    touched[indices] = True
    assert np.array_equal(got[:, ~touched], W0[:, ~touched])
    # and the dense entry points give the same bits
    Wd = dev(W0)
    if signed:
        ctx.sfb_apply_signed(Wd, dev_vals(U, bf16), dev_vals(V, bf16).reshape(N, D), coef_d, eta)
    else:
        ctx.sfb_apply(Wd, dev_vals(U, bf16), dev_vals(V, bf16).reshape(N, D), eta)
    assert torch.equal(W, Wd)


def test_csr_shadow_copy_stays_current(sfb, oracle):
    """CSR calls keep an attached bf16 working copy of W current, like the dense ones."""
    J, D, B, eta = 520, 328, 200, 0.05
    W0 = S.normal_matrix(J, D, 0.05, seed=22)
    ca, cb = sfb.Context(0), sfb.Context(0)
    Wa, Wb = dev(W0), dev(W0)
    ca.sfb_shadow_attach(Wa)
    Ua = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0"); Ub = torch.empty_like(Ua)
    for step in range(3):
        X, y = S.mlr_batch(J, D, B, seed=22, step=step, zero_frac=0.9, bf16=True)
        _, (ip, ix, vals) = csr_dev(X, True)
        ca.sfb_mlr_sf_csr(Wa, ip, ix, vals, dev(y), Ua)
        cb.sfb_mlr_sf_csr(Wb, ip, ix, vals, dev(y), Ub)
        assert torch.equal(Ua, Ub), step
        ca.sfb_apply_csr(Wa, Ua, ip, ix, vals, eta); cb.sfb_apply_csr(Wb, Ub, ip, ix, vals, eta)
        assert torch.equal(Wa, Wb)
    ca.close(); cb.close()


def test_csr_edge_cases_and_check(ctx, sfb):
    J, D = 16, 24
    W = torch.ones((J, D), dtype=torch.float32, device="cuda:0")
    i64 = lambda a: dev(np.array(a, np.int64))
    i32 = lambda a: dev(np.array(a, np.int32))
    f32 = lambda a: dev(np.array(a, np.float32))
    # no rows: nothing happens
    U0 = torch.empty((0, J), dtype=torch.float32, device="cuda:0")
    ctx.sfb_apply_csr(W, U0, i64([0]), i32([]), f32([]), 1.0)
    # rows without entries: W unchanged
    U2 = torch.ones((2, J), dtype=torch.float32, device="cuda:0")
    ctx.sfb_apply_csr(W, U2, i64([0, 0, 0]), i32([]), f32([]), 1.0)
    torch.cuda.synchronize()
    assert torch.equal(W, torch.ones_like(W))
    # format check: good, unsorted, out of range, bad indptr
    assert ctx.sfb_csr_check(i64([0, 2, 3]), i32([1, 5, 0]), f32([1, 2, 3]), D) == 0
    assert ctx.sfb_csr_check(i64([0, 2, 3]), i32([5, 1, 0]), f32([1, 2, 3]), D) == 1
    assert ctx.sfb_csr_check(i64([0, 2, 3]), i32([1, 1, 0]), f32([1, 2, 3]), D) == 1
    assert ctx.sfb_csr_check(i64([0, 2, 3]), i32([1, D, -1]), f32([1, 2, 3]), D) == 2
    assert ctx.sfb_csr_check(i64([0, 4, 3]), i32([1, 2, 3]), f32([1, 2, 3]), D) >= 1
    assert ctx.sfb_csr_check(i64([1, 2, 3]), i32([1, 2, 3]), f32([1, 2, 3]), D) >= 1
    # entries outside the matrix are dropped, the others applied
    W = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    ctx.sfb_apply_csr(W, U2, i64([0, 2, 3]), i32([1, D + 7, -1]), f32([1, 2, 3]), -1.0)
    torch.cuda.synchronize()
    want = torch.zeros_like(W)
    want[:, 1] = 1.0
    assert torch.equal(W, want)
    # dtype of U must match the values; bf16 shapes must be multiples of 8
    with pytest.raises(TypeError):
        ctx.sfb_apply_csr(W, U2.to(torch.bfloat16), i64([0, 0, 0]), i32([]), f32([]), 1.0)
    Wb = torch.zeros((12, 16), dtype=torch.float32, device="cuda:0")
    with pytest.raises(sfb.SfbError) as e:
        ctx.sfb_apply_csr(Wb, torch.zeros((1, 12), dtype=torch.bfloat16, device="cuda:0"), i64([0, 1]), i32([3]),
                          f32([1]).to(torch.bfloat16), 1.0)
    assert e.value.code == sfb.SFB_EINVAL


@pytest.mark.parametrize("bf16", [False, True])
def test_gather_route_edge_cases(ctx, sfb, oracle, bf16):
    """The route over the stored entries on inputs its re-laying has to survive: rows without entries, entries
    outside the matrix (ignored), unsorted columns within a row (the stored entries still sum up), and no stored
    entry at all."""
    J, D, B = 72, 136, 5
    W0 = S.normal_matrix(J, D, 0.2, seed=12)
    if bf16:
        W0 = S.round_to_bf16(W0)
    g = np.random.default_rng(7)
    # row 0: unsorted columns; row 1: empty; row 2: one entry out of range on either side; row 3: last column; row 4: first
    rows = [[(100, 0.5), (3, -1.0), (64, 2.0)], [], [(-1, 9.0), (7, 1.5), (D, 9.0)], [(D - 1, -0.25)], [(0, 1.0)]]
    indptr = np.zeros(B + 1, np.int64)
    idx, val = [], []
    for i, r in enumerate(rows):
        for c, v in r:
            idx.append(c); val.append(v)
        indptr[i + 1] = len(idx)
    idx = np.array(idx, np.int32); val = np.array(val, np.float32)
    y = g.integers(0, J, B).astype(np.int32)
    keep = (idx >= 0) & (idx < D)
    Xd = np.zeros((B, D), np.float32)
    for i in range(B):
        for t in range(indptr[i], indptr[i + 1]):
            if keep[t]:
                Xd[i, idx[t]] += val[t]
    Uo, _ = oracle.mlr_sf(W0, Xd, y)
    dt = torch.bfloat16 if bf16 else torch.float32
    vals = dev(S.bf16_bits(val)).view(torch.bfloat16) if bf16 else dev(val)
    U = torch.empty((B, J), dtype=dt, device="cuda:0")
    ctx.sfb_set_csr_route(2)
    try:
        ctx.sfb_mlr_sf_csr(dev(W0), dev(indptr), dev(idx), vals, dev(y), U)
        assert rel_err(host(U), Uo) <= (TOL_BF16 if bf16 else TOL_F32)
        mlr_u_check(host(U), Uo, y, TOL_BF16 if bf16 else TOL_F32, label_tol=1e-2 if bf16 else None)
        # nothing stored: every logit is zero, every probability 1/J
        U2 = torch.empty_like(U)
        empty_i = torch.zeros((0,), dtype=torch.int32, device="cuda:0")
        empty_v = torch.zeros((0,), dtype=dt, device="cuda:0")
        ctx.sfb_mlr_sf_csr(dev(W0), dev(np.zeros(B + 1, np.int64)), empty_i, empty_v, dev(y), U2)
        want = np.full((B, J), 1.0 / J); want[np.arange(B), y] -= 1.0
        assert rel_err(host(U2), want) <= (TOL_BF16 if bf16 else TOL_F32)
    finally:
        ctx.sfb_set_csr_route(0)
