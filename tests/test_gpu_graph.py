"""The library's calls can be captured into a HIP graph and replayed: a whole sparse-coding step
(about 90 dependent launches) and an MLR step, replayed several times with eager work and
synchronisations in between, must reproduce the eager results bit for bit (the library enqueues
kernels and device-to-device copies only: no memset nodes, no allocation, no host synchronisation)."""
import numpy as np
import pytest
import torch

import sfb_synth as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sfb():
    import paper_1409_5705_amd as m
    m.lib()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def test_sparse_coding_step_replays_from_a_graph(sfb):
    J, D, B = 512, 256, 96
    W0 = dev(S.sc_dictionary(J, D, seed=1))
    X = dev(S.sc_batch(D, B, seed=1))
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = sfb.Context(0)                       # bound to the side stream
        W = W0.clone()
        U = torch.empty((B, J), dtype=torch.float32, device="cuda:0")
        V = torch.empty((B, D), dtype=torch.float32, device="cuda:0")

        def step():
            ctx.sfb_compute_sf(sfb.SFB_SC, W, X, U=U, V=V, lam=0.1, ista_iters=6, power_iters=4)
            ctx.sfb_apply(W, U, V, -0.01)
            ctx.sfb_prox_rows(W, sfb.SFB_PROX_NORMALIZE)

        step()                                      # eager: also sizes the workspace
        side.synchronize()
        ref = [W.clone()]
        for _ in range(3):
            step()
            side.synchronize()
            ref.append(W.clone())
        W.copy_(W0)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for k in range(4):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(W, ref[k]), "replay %d differs from the eager step" % k
        junk = torch.randn(1 << 20, device="cuda:0").sum().item()      # unrelated eager work between replays
        assert np.isfinite(junk)
    ctx.close()


def test_mlr_bf16_step_replays_from_a_graph(sfb):
    J, D, B = 1000, 520, 130
    W0 = dev(S.normal_matrix(J, D, 0.02, seed=2))
    Xh, yh = S.mlr_batch(J, D, B, seed=2, zero_frac=0.9, bf16=True)
    X = dev(S.bf16_bits(Xh)).view(torch.bfloat16)
    y = dev(yh)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = sfb.Context(0)
        W = W0.clone()
        ctx.sfb_shadow_attach(W)
        U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")

        def step():
            ctx.sfb_compute_sf(sfb.SFB_MLR, W, X, Y=y, U=U)
            ctx.sfb_apply(W, U, X, 0.05)

        step()
        side.synchronize()
        ref = [W.clone()]
        for _ in range(2):
            step()
            side.synchronize()
            ref.append(W.clone())
        W.copy_(W0)
        ctx.sfb_shadow_attach(W)                    # refresh the bf16 working copy from the restored W
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(W, ref[k]), "replay %d differs from the eager step" % k
    ctx.close()


def test_mlr_bf16_step_on_split_storage_replays_from_a_graph(sfb):
    """The same step with W kept as two 16-bit planes; the export is part of the captured graph."""
    J, D, B = 1000, 520, 130
    W0 = dev(S.normal_matrix(J, D, 0.02, seed=3))
    Xh, yh = S.mlr_batch(J, D, B, seed=3, zero_frac=0.9, bf16=True)
    X = dev(S.bf16_bits(Xh)).view(torch.bfloat16)
    y = dev(yh)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = sfb.Context(0)
        W = W0.clone()
        ctx.sfb_split_attach(W)
        U = torch.empty((B, J), dtype=torch.bfloat16, device="cuda:0")

        def step():
            ctx.sfb_compute_sf(sfb.SFB_MLR, W, X, Y=y, U=U)
            ctx.sfb_apply(W, U, X, 0.05)
            ctx.sfb_split_export(W)

        step()
        side.synchronize()
        ref = [W.clone()]
        for _ in range(2):
            step()
            side.synchronize()
            ref.append(W.clone())
        W.copy_(W0)
        ctx.sfb_split_attach(W)                     # planes back to the start
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(W, ref[k]), "replay %d differs from the eager step" % k
        junk = torch.randn(1 << 20, device="cuda:0").sum().item()
        assert np.isfinite(junk)
    ctx.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_apply_static_replays_from_a_graph(sfb, dtype):
    """sfb_apply_static is the entry point for callers that cannot allocate: captured on its own (the context never
    gets a workspace), replayed with eager work in between, it must give the bits of eager sfb_apply."""
    J, D, N = (1000, 520, 130) if dtype == "bf16" else (264, 200, 96)
    W0 = dev(S.normal_matrix(J, D, 0.02, seed=4))
    Uh, Vh = S.mlr_peer_sf(J, D, N, seed=4, step=0, peer=0, bf16=(dtype == "bf16"))
    if dtype == "bf16":
        U, V = dev(S.bf16_bits(Uh)).view(torch.bfloat16), dev(S.bf16_bits(Vh)).view(torch.bfloat16)
    else:
        U, V = dev(Uh.astype(np.float32)), dev(Vh.astype(np.float32))
    ref_ctx = sfb.Context(0)
    Wr = W0.clone()
    ref = []
    for _ in range(3):
        ref_ctx.sfb_apply(Wr, U, V, 0.05)
        torch.cuda.synchronize()
        ref.append(Wr.clone())
    ref_ctx.close()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = sfb.Context(0)                        # no workspace is ever set on this context
        W = W0.clone()
        ctx.sfb_apply_static(W0.clone(), U, V, 0.05)     # one eager call first (kernel attributes are set on first use)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ctx.sfb_apply_static(W, U, V, 0.05)
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(W, ref[k]), "replay %d differs from eager sfb_apply" % k
        junk = torch.randn(1 << 20, device="cuda:0").sum().item()
        assert np.isfinite(junk)
    ctx.close()
