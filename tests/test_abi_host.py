"""Host-side checks of the C-ABI library that need no GPU: it loads, it exports
every symbol the header declares, and the argument logic that runs before any
device call behaves as documented."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sfb():
    import paper_1409_5705_amd as m
    if not os.path.exists(m.binding.LIB_PATH):
        from paper_1409_5705_amd.build import build_library
        build_library()
    m.lib()
    return m


def test_exports_every_declared_symbol(sfb):
    hdr = open(os.path.join(ROOT, "include", "sfb.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(sfb_[a-z0-9_]+)\s*\(", hdr)))
    assert {"sfb_create", "sfb_destroy", "sfb_compute_sf", "sfb_apply", "sfb_prox_rows",
            "sfb_workspace_bytes", "sfb_set_workspace", "sfb_strerror"} <= set(names)
    L = sfb.lib()
    for n in names:
        assert hasattr(L, n), n


def test_strerror_and_version(sfb):
    assert sfb.strerror(0) == "success"
    assert "workspace" in sfb.strerror(sfb.SFB_ENOWS)
    assert "invalid" in sfb.strerror(sfb.SFB_EINVAL)
    assert re.match(r"^\d+\.\d+$", sfb.version())


def _batch(sfb, B=8, in_dtype=0, sf_dtype=0, ista=20, power=10, lam=0.1):
    b = sfb.sfb_batch()
    b.B = B
    b.in_dtype = in_dtype
    b.sf_dtype = sf_dtype
    b.ista_iters = ista
    b.power_iters = power
    b.lambda_ = lam
    b.margin = 1.0
    return b


def test_workspace_bytes_logic(sfb):
    L = sfb.lib()
    wb = lambda model, J, D, b: L.sfb_workspace_bytes(model, J, D, ctypes.byref(b))
    assert wb(sfb.SFB_MLR, 100, 64, _batch(sfb, B=8)) >= 8 * 100 * 4
    assert wb(sfb.SFB_MLR, 100, 64, _batch(sfb, B=8)) % 256 == 0
    # bf16 MLR: logits + aligned copy of X + room for a bf16 copy of W
    full = wb(sfb.SFB_MLR, 104, 72, _batch(sfb, B=8, in_dtype=1, sf_dtype=1))
    assert full >= 8 * 104 * 4 + 8 * 128 * 2 + L.sfb_shadow_bytes(104, 72)
    assert L.sfb_shadow_bytes(104, 72) >= 104 * 128 * 2 and L.sfb_shadow_bytes(104, 70) == sfb.SFB_EINVAL
    assert L.sfb_apply_workspace_bytes(104, 72, 10, 1) >= (104 + 72) * 64 * 2
    assert L.sfb_apply_workspace_bytes(104, 72, 10, 0) == 0
    assert wb(sfb.SFB_DML, 16, 64, _batch(sfb, B=4)) >= 4 * 16 * 4
    assert wb(sfb.SFB_SC, 128, 64, _batch(sfb)) > (64 + 128 + 64) * 4
    # bad arguments are reported, not crashed on
    assert wb(sfb.SFB_MLR, 0, 64, _batch(sfb)) == sfb.SFB_EINVAL
    assert wb(7, 10, 64, _batch(sfb)) == sfb.SFB_EINVAL
    assert wb(sfb.SFB_MLR, 100, 64, _batch(sfb, in_dtype=1, sf_dtype=0)) == sfb.SFB_EINVAL
    assert wb(sfb.SFB_MLR, 100, 60, _batch(sfb, in_dtype=1, sf_dtype=1)) == sfb.SFB_EINVAL   # D % 8
    assert wb(sfb.SFB_DML, 16, 64, _batch(sfb, in_dtype=1, sf_dtype=1)) == sfb.SFB_EINVAL    # fp32 only
    assert wb(sfb.SFB_SC, 16, 64, _batch(sfb, power=0)) == sfb.SFB_EINVAL
    assert L.sfb_workspace_bytes(sfb.SFB_MLR, 10, 10, None) == sfb.SFB_EINVAL


def test_sizes_of_the_later_entry_points(sfb):
    L = sfb.lib()
    # high plane: whole blocks of 256 rows x the 128-column pitch; low plane: whole 256 x 256 tiles of 16-bit words
    assert L.sfb_split_bytes(104, 72) == 256 * 128 * 2 + 256 * 256 * 2 and L.sfb_split_bytes(104, 70) == sfb.SFB_EINVAL
    # CSR: bf16 needs no more than the dense call, fp32 a dense copy of X (or V) more
    b16 = _batch(sfb, B=8, in_dtype=1, sf_dtype=1)
    assert L.sfb_mlr_sf_csr_workspace_bytes(104, 72, 8, 1) == L.sfb_workspace_bytes(sfb.SFB_MLR, 104, 72, ctypes.byref(b16))
    b32 = _batch(sfb, B=8)
    assert L.sfb_mlr_sf_csr_workspace_bytes(104, 72, 8, 0) >= L.sfb_workspace_bytes(sfb.SFB_MLR, 104, 72, ctypes.byref(b32)) + 8 * 72 * 4
    assert L.sfb_apply_csr_workspace_bytes(104, 72, 10, 1) == L.sfb_apply_workspace_bytes(104, 72, 10, 1)
    assert L.sfb_apply_csr_workspace_bytes(104, 72, 10, 0) >= 10 * 72 * 4
    assert L.sfb_apply_signed_workspace_bytes(104, 72, 10, 0) >= 10 * 72 * 4
    assert L.sfb_mlr_sf_csr_workspace_bytes(104, 72, 8, 5) == sfb.SFB_EINVAL
    # SDCA: logits of the batch
    assert L.sfb_sdca_workspace_bytes(100, 64, 8) >= 8 * 100 * 4 and L.sfb_sdca_workspace_bytes(0, 64, 8) == sfb.SFB_EINVAL
    # calls on a null context
    assert L.sfb_split_detach(None) == sfb.SFB_EINVAL and L.sfb_split_export(None, None) == sfb.SFB_EINVAL
    assert L.sfb_csr_check(None, None, None) == sfb.SFB_EINVAL
    assert L.sfb_sdca_mlr_sf(None, None, 4, 4, None, 1, None, ctypes.c_float(0.1), 10, ctypes.c_float(1.0), None) == sfb.SFB_EINVAL


def test_null_context_is_rejected(sfb):
    L = sfb.lib()
    assert L.sfb_apply(None, None, 4, 4, None, None, 1, 0, ctypes.c_float(0.1)) == sfb.SFB_EINVAL
    assert L.sfb_prox_rows(None, None, 4, 4, 0) == sfb.SFB_EINVAL
    assert L.sfb_destroy(None) == sfb.SFB_EINVAL
    assert L.sfb_create(None, 0, None) == sfb.SFB_EINVAL


def test_product_never_imports_oracle():
    pkg = os.path.join(ROOT, "paper_1409_5705_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt.lower(), os.path.join(dirpath, f)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            txt = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_1409_5705_amd" not in txt and "libsfb.so" not in txt
