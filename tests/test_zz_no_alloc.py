"""sfb_apply_static (the entry point for callers that cannot allocate: its scratch is a static device array
inside the library) against sfb_apply, through the C-ABI: two calls in a row on the shared array, the second
with a smaller input, same bits as the entry point that works in the caller's workspace; no workspace set on
the context that makes the static calls; too large a shape is refused."""
import ctypes

import numpy as np
import pytest

import sfb_synth as S

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


def _factors(J, D, N, bf16, seed):
    U, V = S.mlr_peer_sf(J, D, N, seed=seed, step=0, peer=0, bf16=bf16)
    if bf16:
        return dev(S.bf16_bits(U)).view(torch.bfloat16), dev(S.bf16_bits(V)).view(torch.bfloat16), U, V
    return dev(U), dev(V), U, V


@pytest.mark.parametrize("bf16,shapes", [
    (True, [(1024, 1000, 2056), (130, 264, 136)]),       # U^T, V^T of the bf16 contraction in the static array
    (False, [(1024, 200, 136), (512, 64, 96)]),          # k-split partial sums of the fp32 contraction
])
def test_apply_static_matches_apply(sfb, oracle, bf16, shapes):
    from parity import TOL_F32, trajectory_check
    L = sfb.lib()
    dt = sfb.SFB_BF16 if bf16 else sfb.SFB_F32
    ref_ctx = sfb.Context(0)                  # works in a torch-allocated workspace
    st_ctx = sfb.Context(0)                   # never given a workspace
    for call, (N, J, D) in enumerate(shapes):
        print("apply_static", "bf16" if bf16 else "f32", N, J, D, flush=True)
        assert 0 < L.sfb_apply_workspace_bytes(J, D, N, dt) <= sfb.SFB_STATIC_SCRATCH_BYTES
        Ud, Vd, U, V = _factors(J, D, N, bf16, seed=40 + call)
        W0 = S.normal_matrix(J, D, 0.01, seed=41 + call)
        Wa, Wb = dev(W0), dev(W0)
        ref_ctx.sfb_apply(Wa, Ud, Vd, 0.01)
        rc = L.sfb_apply_static(st_ctx._h, Wb.data_ptr(), J, D, Ud.data_ptr(), Vd.data_ptr(), N, dt, ctypes.c_float(0.01))
        assert rc == sfb.SFB_OK, (rc, sfb.strerror(rc), L.sfb_last_hip_error(st_ctx._h))
        torch.cuda.synchronize()
        assert torch.equal(Wa, Wb)            # the same kernels on the same operands: the same bits
        ref = oracle.apply(W0, U, V, 0.01)
        trajectory_check(Wb.cpu().numpy(), ref, W0, 1, TOL_F32)
    assert st_ctx._ws is None
    # beyond the array: refused, W untouched
    N, J, D = 4096, 8192, 4096
    assert L.sfb_apply_workspace_bytes(J, D, N, sfb.SFB_BF16) > sfb.SFB_STATIC_SCRATCH_BYTES
    W = torch.zeros((J, D), dtype=torch.float32, device="cuda:0")
    Ud = torch.zeros((N, J), dtype=torch.bfloat16, device="cuda:0")
    Vd = torch.ones((N, D), dtype=torch.bfloat16, device="cuda:0")
    rc = L.sfb_apply_static(st_ctx._h, W.data_ptr(), J, D, Ud.data_ptr(), Vd.data_ptr(), N, sfb.SFB_BF16,
                            ctypes.c_float(1.0))
    assert rc == sfb.SFB_ETOOBIG
    assert "static scratch" in sfb.strerror(rc)
    with pytest.raises(sfb.SfbError) as e:
        st_ctx.sfb_apply_static(W, Ud, Vd, 1.0)
    assert e.value.code == sfb.SFB_ETOOBIG
    torch.cuda.synchronize()
    assert float(W.abs().max()) == 0.0
    ref_ctx.close(); st_ctx.close()
