"""GPU parity at the full size of the headline workload (MLR, J=325,000 classes,
D=10,000 features, B=1024, bf16 inputs, fp32 W), in the launch configuration the
bench times (W kept as two 16-bit planes, sfb_split_attach).  The oracle cannot finish the whole step in seconds, so:

 * SFs: all J entries of u for a few sampled samples, computed one by one by the
   oracle from the same W and X;
 * reconstruction: sfb_apply on W = 0 with generated factors, compared on a
   random subset of rows of W (the oracle's apply is separable over rows);
 * a whole-matrix property that holds at any size: column sums of the update
   equal sum_i (sum_j U[i][j]) V[i][d].
"""
import numpy as np
import pytest

import sfb_synth as S
from parity import TOL_BF16, TOL_F32, mlr_u_check, rel_err, trajectory_check

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

CFG = S.CONFIGS["mlr_large_bf16"]


@pytest.fixture(scope="module")
def sfb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1409_5705_amd as m
    m.lib()
    return m


@pytest.fixture(scope="module")
def big(sfb):
    J, D, B = CFG["J"], CFG["D"], CFG["B"]
    print("large: generating W on device", flush=True)
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(0)
    W = torch.randn((J, D), dtype=torch.float32, device="cuda:0", generator=gen) * CFG["sigma"]
    X, y = S.mlr_batch(J, D, B, seed=0, zero_frac=CFG["zero_frac"], bf16=True)
    Xd = torch.from_numpy(S.bf16_bits(X)).to("cuda:0").view(torch.bfloat16)
    yd = torch.from_numpy(y).to("cuda:0")
    ctx = sfb.Context(0)
    ctx.sfb_split_attach(W)       # the configuration the bench times: W as two 16-bit planes
    yield dict(W=W, X=X, y=y, Xd=Xd, yd=yd, ctx=ctx, J=J, D=D, B=B)
    ctx.close()


@pytest.mark.timeout(600)
def test_large_mlr_sf_sampled(big, sfb, oracle):
    J, D, B = big["J"], big["D"], big["B"]
    U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
    print("large: compute_sf", flush=True)
    big["ctx"].sfb_compute_sf(sfb.SFB_MLR, big["W"], big["Xd"], Y=big["yd"], U=U)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 255, 256, 300, 511, 512, 700, 767, 768, 1022, 1023])      # every 256-sample tile, both its ends
    print("large: W to host", flush=True)
    Wh = big["W"].cpu().numpy()
    print("large: oracle on %d samples" % len(rows), flush=True)
    Uo, _ = oracle.mlr_sf(Wh, big["X"][rows], big["y"][rows])
    del Wh
    Ug = U[torch.from_numpy(rows).to("cuda:0")].float().cpu().numpy()
    err = rel_err(Ug, Uo)
    print("large: U err", err, flush=True)
    assert err <= TOL_BF16
    # all J classes of the sampled rows (every class tile), label entry apart: probabilities of ~3e-6 against
    # their own rms, plus each row's least-squares factor
    merr = mlr_u_check(Ug, Uo, big["y"][rows], TOL_BF16, factor_tol=1e-3, label_tol=1e-2)
    print("large: U err with the label entry masked", merr, flush=True)
    # the label entry and the zero-sum property on every sample (bf16 rounding of ~3e-6 entries)
    s = U.float().sum(dim=1).cpu().numpy()
    assert np.max(np.abs(s)) < 2e-2
    big["U"] = U


@pytest.mark.timeout(600)
def test_large_apply_reconstruction(big, sfb, oracle):
    J, D, B = big["J"], big["D"], big["B"]
    print("large: generating factors", flush=True)
    g = np.random.default_rng(11)
    # U with the magnitude mix of MLR factors: ~1/J everywhere, -1 at one label per row
    Uh = (g.random((B, J), dtype=np.float32) * np.float32(2.0 / J))
    Uh[np.arange(B), g.integers(0, J, B)] -= 1.0
    Uh = S.round_to_bf16(Uh)
    Ud = torch.from_numpy(S.bf16_bits(Uh)).to("cuda:0").view(torch.bfloat16)
    Wz = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    print("large: apply (on the two planes, as the bench does; then export)", flush=True)
    c2 = sfb.Context(0)
    c2.sfb_split_attach(Wz)
    c2.sfb_apply(Wz, Ud, big["Xd"], 1.0)
    c2.sfb_split_export(Wz)
    torch.cuda.synchronize()
    print("large: apply on an fp32 array", flush=True)
    Wf = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    big["ctx"].sfb_apply(Wf, Ud, big["Xd"], 1.0)
    torch.cuda.synchronize()
    assert torch.equal(Wz, Wf)                       # same bits in either storage
    del Wf
    rows = np.sort(g.choice(J, size=1536, replace=False))
    rows[:4] = [0, 1, 2, 3]; rows[-4:] = [J - 4, J - 3, J - 2, J - 1]
    rows = np.unique(rows)
    print("large: oracle apply on %d rows" % len(rows), flush=True)
    ref = oracle.apply(np.zeros((len(rows), D)), Uh[:, rows], big["X"], 1.0)
    got = Wz[torch.from_numpy(rows).to("cuda:0")].cpu().numpy()
    err = rel_err(got, ref)
    print("large: reconstruction err", err, flush=True)
    assert err <= TOL_F32
    # whole-matrix property: column sums
    colsum = Wz.sum(dim=0, dtype=torch.float64)
    s = Ud.double().sum(dim=1)
    expect = -(s @ big["Xd"].double())
    e2 = float((colsum - expect).abs().max() / expect.abs().max())
    print("large: column-sum err", e2, flush=True)
    assert e2 < 1e-3
    # second application with the opposite sign restores zero (up to rounding of the sums)
    c2.sfb_apply(Wz, Ud, big["Xd"], -1.0)
    c2.sfb_split_export(Wz)
    torch.cuda.synchronize()
    assert float(Wz.abs().max()) == 0.0
    c2.close()


@pytest.mark.timeout(600)
def test_large_csr_entry_points_match_dense(big, sfb):
    """At full size the CSR entry points (samples and second factors as stored non-zeros) give the
    bits of the dense ones, whose results the two tests above compare with the oracle."""
    J, D, B = big["J"], big["D"], big["B"]
    indptr, indices, values = S.csr_from_dense(big["X"])
    print("large: csr nnz %d (density %.3f)" % (len(indices), len(indices) / (B * D)), flush=True)
    ip = torch.from_numpy(indptr).to("cuda:0")
    ix = torch.from_numpy(indices).to("cuda:0")
    vals = torch.from_numpy(S.bf16_bits(values)).to("cuda:0").view(torch.bfloat16)
    ctx = big["ctx"]
    assert ctx.sfb_csr_check(ip, ix, vals, D) == 0
    U = big.get("U")
    if U is None:
        U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
        ctx.sfb_compute_sf(sfb.SFB_MLR, big["W"], big["Xd"], Y=big["yd"], U=U)
    U2 = torch.empty_like(U)
    print("large: mlr_sf_csr", flush=True)
    ctx.sfb_mlr_sf_csr(big["W"], ip, ix, vals, big["yd"], U2)
    torch.cuda.synchronize()
    assert torch.equal(U, U2)
    Wa = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    Wb = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    print("large: apply dense / csr", flush=True)
    ctx.sfb_apply(Wa, U, big["Xd"], 1.0)
    ctx.sfb_apply_csr(Wb, U, ip, ix, vals, 1.0)
    torch.cuda.synchronize()
    assert torch.equal(Wa, Wb)


@pytest.mark.timeout(600)
def test_large_trajectory_reduced_d(sfb, oracle):
    """The headline workload's 5 steps (eta = 0.001) with all 325,000 classes on the two planes, at a feature
    count the host oracle can carry (D = 200: k ragged against the 64-wide slices; B = 512): SF computation and
    application alternate, the oracle keeps W in fp64, factors and the final W are compared."""
    J, B, eta, steps = CFG["J"], CFG["B"] // 2, CFG["eta"], CFG["steps"]
    D = 200
    W0 = S.normal_matrix(J, D, CFG["sigma"], seed=2)
    W = torch.from_numpy(W0).to("cuda:0")
    c = sfb.Context(0)
    c.sfb_split_attach(W)
    Wo = W0.astype(np.float64)
    U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
    for step in range(steps):
        X, y = S.mlr_batch(J, D, B, seed=2, step=step, zero_frac=CFG["zero_frac"], bf16=True)
        Xd = torch.from_numpy(S.bf16_bits(X)).to("cuda:0").view(torch.bfloat16)
        c.sfb_compute_sf(sfb.SFB_MLR, W, Xd, Y=torch.from_numpy(y).to("cuda:0"), U=U)
        c.sfb_apply(W, U, Xd, eta)
        torch.cuda.synchronize()
        Uo, _ = oracle.mlr_sf(Wo, X, y)
        err = mlr_u_check(U.float().cpu().numpy(), Uo, y, TOL_BF16, factor_tol=1e-3, label_tol=1e-2)
        print("large trajectory: step", step, "masked U err", err, flush=True)
        Wo = oracle.apply(Wo, Uo, X, eta)
    c.sfb_split_export(W)
    torch.cuda.synchronize()
    trajectory_check(W.cpu().numpy(), Wo, W0, steps, TOL_BF16)
    c.close()


@pytest.mark.timeout(600)
def test_large_csr_forward_over_stored_entries(big, sfb, oracle):
    """At the headline shape with tf-idf-like sparsity (0.5 % of the features non-zero) sfb_mlr_sf_csr goes over
    the stored entries (W streamed once); its factors against the oracle's loop over the same entries on sampled
    rows, and against the dense route on all of them."""
    J, D, B = big["J"], big["D"], big["B"]
    X, y = S.mlr_batch(J, D, B, seed=3, zero_frac=0.995, bf16=True)
    indptr, indices, values = S.csr_from_dense(X)
    ip = torch.from_numpy(indptr).to("cuda:0")
    ix = torch.from_numpy(indices).to("cuda:0")
    vals = torch.from_numpy(S.bf16_bits(values)).to("cuda:0").view(torch.bfloat16)
    yd = torch.from_numpy(y).to("cuda:0")
    ctx = big["ctx"]
    Ug = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")
    Ud = torch.empty_like(Ug)
    ctx.sfb_profile_enable(True)
    ctx.sfb_profile_collect()
    ctx.sfb_mlr_sf_csr(big["W"], ip, ix, vals, yd, Ug)              # route left to the library
    ran = ctx.sfb_profile_collect()
    ctx.sfb_profile_enable(False)
    print("large csr: kernels", ran, flush=True)
    assert "csr_forward_gather" in ran
    ctx.sfb_set_csr_route(1)
    ctx.sfb_mlr_sf_csr(big["W"], ip, ix, vals, yd, Ud)
    ctx.sfb_set_csr_route(0)
    torch.cuda.synchronize()
    same = float((Ug == Ud).float().mean())
    print("large csr: entries identical to the dense route's: %.5f" % same, flush=True)
    assert same > 0.99
    rows = np.array([0, 255, 256, 511, 700, 1023])
    Wh = big["W"].cpu().numpy()
    sub_ptr = np.zeros(len(rows) + 1, dtype=np.int64)
    sub_idx, sub_val = [], []
    for k, r in enumerate(rows):
        sub_idx.append(indices[indptr[r]:indptr[r + 1]]); sub_val.append(values[indptr[r]:indptr[r + 1]])
        sub_ptr[k + 1] = sub_ptr[k] + len(sub_idx[-1])
    Uo = oracle.mlr_sf_csr(Wh, sub_ptr, np.concatenate(sub_idx), np.concatenate(sub_val), y[rows])
    del Wh
    got = Ug[torch.from_numpy(rows).to("cuda:0")].float().cpu().numpy()
    err = mlr_u_check(got, Uo, y[rows], TOL_BF16, factor_tol=1e-3, label_tol=1e-2)
    print("large csr: masked U err", err, flush=True)
