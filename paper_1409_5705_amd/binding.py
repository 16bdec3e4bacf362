"""ctypes binding of libsfb's C-ABI (include/sfb.h).

Argument marshalling only: torch tensors supply device memory and the stream;
every step of the path runs in the library's kernels.  There is no fallback:
if the shared library is missing, importing this module's functions raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsfb.so")

SFB_MLR, SFB_DML, SFB_SC = 0, 1, 2
SFB_F32, SFB_BF16 = 0, 1
SFB_PROX_PROJECT, SFB_PROX_NORMALIZE = 0, 1
SFB_OK, SFB_EINVAL, SFB_ENOWS, SFB_EHIP, SFB_ETOOBIG = 0, -1, -2, -3, -4
SFB_STATIC_SCRATCH_BYTES = 32 << 20


class sfb_batch(ctypes.Structure):
    _fields_ = [
        ("X", ctypes.c_void_p),
        ("Y", ctypes.c_void_p),
        ("sim", ctypes.c_void_p),
        ("B", ctypes.c_int64),
        ("in_dtype", ctypes.c_int32),
        ("sf_dtype", ctypes.c_int32),
        ("lambda_", ctypes.c_float),
        ("ista_iters", ctypes.c_int32),
        ("power_iters", ctypes.c_int32),
        ("margin", ctypes.c_float),
    ]


class sfb_csr(ctypes.Structure):
    _fields_ = [
        ("indptr", ctypes.c_void_p),
        ("indices", ctypes.c_void_p),
        ("values", ctypes.c_void_p),
        ("rows", ctypes.c_int64),
        ("cols", ctypes.c_int64),
        ("nnz", ctypes.c_int64),
        ("dtype", ctypes.c_int32),
    ]


class sfb_kernel_time(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("launches", ctypes.c_int32), ("total_ms", ctypes.c_float)]


class SfbError(RuntimeError):
    def __init__(self, code, what, hip=0):
        self.code = code
        self.hip = hip
        super().__init__("%s failed: %d (%s)%s" % (what, code, strerror(code), " hip=%d" % hip if hip else ""))


_lib = None


def lib():
    """The loaded C library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libsfb.so is not built (%s); run __graft_entry__.build() or "
                "python paper_1409_5705_amd/build.py" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        L.sfb_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, vp]
        L.sfb_create.restype = ctypes.c_int
        L.sfb_destroy.argtypes = [vp]
        L.sfb_destroy.restype = ctypes.c_int
        L.sfb_workspace_bytes.argtypes = [i32, i64, i64, ctypes.POINTER(sfb_batch)]
        L.sfb_workspace_bytes.restype = i64
        L.sfb_apply_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.sfb_apply_workspace_bytes.restype = i64
        L.sfb_shadow_bytes.argtypes = [i64, i64]
        L.sfb_shadow_bytes.restype = i64
        L.sfb_shadow_attach.argtypes = [vp, vp, i64, i64, vp, i64]
        L.sfb_shadow_attach.restype = ctypes.c_int
        L.sfb_shadow_detach.argtypes = [vp]
        L.sfb_shadow_detach.restype = ctypes.c_int
        L.sfb_split_bytes.argtypes = [i64, i64]
        L.sfb_split_bytes.restype = i64
        L.sfb_split_attach.argtypes = [vp, vp, i64, i64, vp, i64]
        L.sfb_split_attach.restype = ctypes.c_int
        L.sfb_split_export.argtypes = [vp, vp]
        L.sfb_split_export.restype = ctypes.c_int
        L.sfb_split_detach.argtypes = [vp]
        L.sfb_split_detach.restype = ctypes.c_int
        L.sfb_set_workspace.argtypes = [vp, vp, i64]
        L.sfb_set_workspace.restype = ctypes.c_int
        L.sfb_compute_sf.argtypes = [vp, i32, vp, i64, i64, ctypes.POINTER(sfb_batch), vp, vp, vp]
        L.sfb_compute_sf.restype = ctypes.c_int
        L.sfb_apply.argtypes = [vp, vp, i64, i64, vp, vp, i64, i32, ctypes.c_float]
        L.sfb_apply.restype = ctypes.c_int
        L.sfb_apply_static.argtypes = [vp, vp, i64, i64, vp, vp, i64, i32, ctypes.c_float]
        L.sfb_apply_static.restype = ctypes.c_int
        L.sfb_apply_signed_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.sfb_apply_signed_workspace_bytes.restype = i64
        L.sfb_apply_signed.argtypes = [vp, vp, i64, i64, vp, vp, vp, i64, i32, ctypes.c_float]
        L.sfb_apply_signed.restype = ctypes.c_int
        L.sfb_csr_check.argtypes = [vp, ctypes.POINTER(sfb_csr), ctypes.POINTER(i64)]
        L.sfb_csr_check.restype = ctypes.c_int
        L.sfb_mlr_sf_csr_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.sfb_mlr_sf_csr_workspace_bytes.restype = i64
        L.sfb_mlr_sf_csr.argtypes = [vp, vp, i64, i64, ctypes.POINTER(sfb_csr), vp, vp]
        L.sfb_mlr_sf_csr.restype = ctypes.c_int
        L.sfb_set_csr_route.argtypes = [vp, ctypes.c_int]
        L.sfb_set_csr_route.restype = ctypes.c_int
        L.sfb_apply_csr_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.sfb_apply_csr_workspace_bytes.restype = i64
        L.sfb_apply_csr.argtypes = [vp, vp, i64, i64, vp, ctypes.POINTER(sfb_csr), vp, ctypes.c_float]
        L.sfb_apply_csr.restype = ctypes.c_int
        L.sfb_sdca_workspace_bytes.argtypes = [i64, i64, i64]
        L.sfb_sdca_workspace_bytes.restype = i64
        L.sfb_sdca_mlr_sf.argtypes = [vp, vp, i64, i64, vp, i64, vp, ctypes.c_float, i64, ctypes.c_float, vp]
        L.sfb_sdca_mlr_sf.restype = ctypes.c_int
        L.sfb_dual_to_primal_l2.argtypes = [vp, vp, vp, i64, i64, ctypes.c_float]
        L.sfb_dual_to_primal_l2.restype = ctypes.c_int
        L.sfb_prox_rows.argtypes = [vp, vp, i64, i64, i32]
        L.sfb_prox_rows.restype = ctypes.c_int
        L.sfb_strerror.argtypes = [ctypes.c_int]
        L.sfb_strerror.restype = ctypes.c_char_p
        L.sfb_last_hip_error.argtypes = [vp]
        L.sfb_last_hip_error.restype = ctypes.c_int
        L.sfb_version.argtypes = []
        L.sfb_version.restype = ctypes.c_char_p
        L.sfb_profile_enable.argtypes = [vp, ctypes.c_int]
        L.sfb_profile_enable.restype = ctypes.c_int
        L.sfb_profile_collect.argtypes = [vp, ctypes.POINTER(sfb_kernel_time), ctypes.c_int,
                                          ctypes.POINTER(ctypes.c_int)]
        L.sfb_profile_collect.restype = ctypes.c_int
        L.sfb_set_wait_limit.argtypes = [vp, ctypes.c_int]
        L.sfb_set_wait_limit.restype = ctypes.c_int
        L.sfb_wait_fallbacks.argtypes = [vp, ctypes.POINTER(i64)]
        L.sfb_wait_fallbacks.restype = ctypes.c_int
        L.sfb_ssp_create.argtypes = [ctypes.POINTER(vp), i32, i32]
        L.sfb_ssp_create.restype = ctypes.c_int
        L.sfb_ssp_destroy.argtypes = [vp]
        L.sfb_ssp_destroy.restype = ctypes.c_int
        L.sfb_ssp_can_compute.argtypes = [vp, i32]
        L.sfb_ssp_can_compute.restype = ctypes.c_int
        L.sfb_ssp_computed.argtypes = [vp, i32]
        L.sfb_ssp_computed.restype = i64
        L.sfb_ssp_delivered.argtypes = [vp, i32, i32]
        L.sfb_ssp_delivered.restype = i64
        L.sfb_ssp_pop_apply.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i64)]
        L.sfb_ssp_pop_apply.restype = ctypes.c_int
        L.sfb_ssp_clock.argtypes = [vp, i32]
        L.sfb_ssp_clock.restype = i64
        L.sfb_ssp_tau.argtypes = [vp, i32, i32]
        L.sfb_ssp_tau.restype = i64
        L.sfb_ssp_arrived.argtypes = [vp, i32, i32]
        L.sfb_ssp_arrived.restype = i64
        L.sfb_ssp_max_staleness_seen.argtypes = [vp]
        L.sfb_ssp_max_staleness_seen.restype = i64
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().sfb_strerror(int(code)).decode()


def version() -> str:
    return lib().sfb_version().decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SFB_F32
    if t.dtype == torch.bfloat16:
        return SFB_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _ptr(t, name, dtype=None, shape=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous (dense row-major)" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %r, got %r" % (name, tuple(shape), tuple(t.shape)))
    return t.data_ptr()


class Context:
    """One sfb_ctx bound to a device and a stream; owns a torch workspace tensor."""

    def __init__(self, device=0, stream=None):
        self._h = ctypes.c_void_p()
        self.device = torch.device("cuda", device) if isinstance(device, int) else torch.device(device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        self.stream = stream
        rc = lib().sfb_create(ctypes.byref(self._h), self.device.index or 0, ctypes.c_void_p(stream.cuda_stream))
        if rc != SFB_OK:
            raise SfbError(rc, "sfb_create")
        self._ws = None
        self._shadow = None          # (W tensor, buffer tensor)

    # -- bf16 working copy of W ----------------------------------------------
    def sfb_shadow_attach(self, W):
        """Allocates (once) and fills the bf16 working copy of W; call again to refresh it."""
        J, D = W.shape
        need = lib().sfb_shadow_bytes(J, D)
        if need < 0:
            raise SfbError(int(need), "sfb_shadow_bytes")
        buf = self._shadow[1] if self._shadow is not None and self._shadow[1].numel() >= need else \
            torch.empty(need, dtype=torch.uint8, device=self.device)
        self._check(lib().sfb_shadow_attach(self._h, _ptr(W, "W", dtype=torch.float32), J, D, buf.data_ptr(),
                                            buf.numel()), "sfb_shadow_attach")
        self._shadow = (W, buf)

    def sfb_shadow_detach(self):
        self._check(lib().sfb_shadow_detach(self._h), "sfb_shadow_detach")
        self._shadow = None

    # -- W kept as two 16-bit planes --------------------------------------------
    def sfb_split_attach(self, W):
        """Allocates (once) the two planes and converts W into them; from then on W's fp32 array is stale
        until sfb_split_export.  Call again to re-convert after changing W yourself."""
        J, D = W.shape
        need = lib().sfb_split_bytes(J, D)
        if need < 0:
            raise SfbError(int(need), "sfb_split_bytes")
        buf = self._shadow[1] if self._shadow is not None and self._shadow[1].numel() >= need else \
            torch.empty(need, dtype=torch.uint8, device=self.device)
        self._check(lib().sfb_split_attach(self._h, _ptr(W, "W", dtype=torch.float32), J, D, buf.data_ptr(),
                                           buf.numel()), "sfb_split_attach")
        self._shadow = (W, buf)

    def sfb_split_export(self, W):
        """Enqueues the write-back of the current parameters into W's fp32 array."""
        self._check(lib().sfb_split_export(self._h, _ptr(W, "W", dtype=torch.float32)), "sfb_split_export")

    def sfb_split_detach(self):
        self._check(lib().sfb_split_detach(self._h), "sfb_split_detach")
        self._shadow = None

    def close(self):
        if self._h:
            lib().sfb_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, what):
        if rc != SFB_OK:
            raise SfbError(rc, what, lib().sfb_last_hip_error(self._h))

    # -- the bounded wait of the softmax of long rows ----------------------------
    def sfb_set_wait_limit(self, polls: int = -1):
        self._check(lib().sfb_set_wait_limit(self._h, int(polls)), "sfb_set_wait_limit")

    def sfb_wait_fallbacks(self) -> int:
        """Partner pairs workgroups computed themselves so far on this device (waits for the stream)."""
        n = ctypes.c_int64(0)
        self._check(lib().sfb_wait_fallbacks(self._h, ctypes.byref(n)), "sfb_wait_fallbacks")
        return int(n.value)

    # -- per-kernel timing ---------------------------------------------------
    def sfb_profile_enable(self, on=True):
        self._check(lib().sfb_profile_enable(self._h, 1 if on else 0), "sfb_profile_enable")

    def sfb_profile_collect(self):
        """Synchronises the stream; returns {kernel group: (launches, total_ms)} since the last collect."""
        buf = (sfb_kernel_time * 32)()
        n = ctypes.c_int(0)
        self._check(lib().sfb_profile_collect(self._h, buf, 32, ctypes.byref(n)), "sfb_profile_collect")
        return {buf[i].name.decode(): (int(buf[i].launches), float(buf[i].total_ms)) for i in range(n.value)}

    # -- workspace ---------------------------------------------------------
    def sfb_workspace_bytes(self, model, J, D, batch: sfb_batch) -> int:
        n = lib().sfb_workspace_bytes(model, J, D, ctypes.byref(batch))
        if n < 0:
            raise SfbError(int(n), "sfb_workspace_bytes")
        return int(n)

    def sfb_set_workspace(self, tensor):
        """Use `tensor` (uint8, device) as scratch; None clears it."""
        if tensor is None:
            self._check(lib().sfb_set_workspace(self._h, None, 0), "sfb_set_workspace")
        else:
            self._check(lib().sfb_set_workspace(self._h, tensor.data_ptr(), tensor.numel() * tensor.element_size()),
                        "sfb_set_workspace")
        self._ws = tensor

    def sfb_apply_workspace_bytes(self, J, D, N, sf_dtype) -> int:
        n = lib().sfb_apply_workspace_bytes(J, D, N, sf_dtype)
        if n < 0:
            raise SfbError(int(n), "sfb_apply_workspace_bytes")
        return int(n)

    def _grow_workspace(self, need):
        have = 0 if self._ws is None else self._ws.numel()
        if need > have:
            self.sfb_set_workspace(torch.empty(need, dtype=torch.uint8, device=self.device))

    def _ensure_workspace(self, model, J, D, batch, W=None):
        need = self.sfb_workspace_bytes(model, J, D, batch)
        if (model == SFB_MLR and batch.in_dtype == SFB_BF16 and self._shadow is not None and W is not None
                and self._shadow[0].data_ptr() == W.data_ptr() and tuple(self._shadow[0].shape) == (J, D)):
            need -= lib().sfb_shadow_bytes(J, D)
        have = 0 if self._ws is None else self._ws.numel()
        if need > have:
            self.sfb_set_workspace(torch.empty(need, dtype=torch.uint8, device=self.device))

    # -- the calls of the path --------------------------------------------
    def sfb_compute_sf(self, model, W, X, Y=None, sim=None, U=None, V=None, n_active=None,
                       lam=0.1, ista_iters=20, power_iters=10, margin=1.0):
        """Enqueues the SF computation; U (and V) must be preallocated device tensors."""
        J, D = W.shape
        B = X.shape[0]
        b = sfb_batch()
        b.X = _ptr(X, "X", shape=(B, D))
        b.B = B
        b.in_dtype = _dtype_code(X)
        b.sf_dtype = _dtype_code(U)
        b.lambda_ = lam
        b.ista_iters = ista_iters
        b.power_iters = power_iters
        b.margin = margin
        if model == SFB_MLR:
            b.Y = _ptr(Y, "Y (labels)", dtype=torch.int32, shape=(B,))
        elif model == SFB_DML:
            b.Y = _ptr(Y, "Y", dtype=X.dtype, shape=(B, D))
            b.sim = _ptr(sim, "sim", dtype=torch.int8, shape=(B,))
        self._ensure_workspace(model, J, D, b, W)
        rc = lib().sfb_compute_sf(self._h, model, _ptr(W, "W", dtype=torch.float32), J, D, ctypes.byref(b),
                                  _ptr(U, "U", shape=(B, J)),
                                  _ptr(V, "V", shape=(B, D)) if V is not None else None,
                                  _ptr(n_active, "n_active", dtype=torch.int32) if n_active is not None else None)
        self._check(rc, "sfb_compute_sf")

    def sfb_apply(self, W, U, V, eta):
        """Enqueues W -= eta * U^T V (in place)."""
        J, D = W.shape
        N = U.shape[0]
        if U.dtype != V.dtype:
            raise TypeError("U and V must share a dtype")
        self._grow_workspace(self.sfb_apply_workspace_bytes(J, D, N, _dtype_code(U)))
        rc = lib().sfb_apply(self._h, _ptr(W, "W", dtype=torch.float32), J, D, _ptr(U, "U", shape=(N, J)),
                             _ptr(V, "V", shape=(N, D)), N, _dtype_code(U), float(eta))
        self._check(rc, "sfb_apply")

    def sfb_apply_static(self, W, U, V, eta):
        """sfb_apply on the library's static scratch: no workspace, nothing allocated (here or in the library)."""
        J, D = W.shape
        N = U.shape[0]
        if U.dtype != V.dtype:
            raise TypeError("U and V must share a dtype")
        rc = lib().sfb_apply_static(self._h, _ptr(W, "W", dtype=torch.float32), J, D, _ptr(U, "U", shape=(N, J)),
                                    _ptr(V, "V", shape=(N, D)), N, _dtype_code(U), float(eta))
        self._check(rc, "sfb_apply_static")

    def sfb_apply_signed(self, W, U, V, coef, eta):
        """Enqueues W -= eta * sum_i coef_i u_i v_i^T (in place); coef: fp32 device tensor [N]."""
        J, D = W.shape
        N = U.shape[0]
        if U.dtype != V.dtype:
            raise TypeError("U and V must share a dtype")
        need = lib().sfb_apply_signed_workspace_bytes(J, D, N, _dtype_code(U))
        if need < 0:
            raise SfbError(int(need), "sfb_apply_signed_workspace_bytes")
        self._grow_workspace(int(need))
        rc = lib().sfb_apply_signed(self._h, _ptr(W, "W", dtype=torch.float32), J, D, _ptr(U, "U", shape=(N, J)),
                                    _ptr(V, "V", shape=(N, D)), _ptr(coef, "coef", dtype=torch.float32, shape=(N,)),
                                    N, _dtype_code(U), float(eta))
        self._check(rc, "sfb_apply_signed")

    # -- CSR rows (samples / second factors) ----------------------------------
    @staticmethod
    def _csr(indptr, indices, values, cols):
        """sfb_csr over three device tensors: int64 [rows + 1], int32 [nnz], fp32 or bf16 [nnz]."""
        m = sfb_csr()
        rows = indptr.numel() - 1
        nnz = indices.numel()
        m.indptr = _ptr(indptr, "indptr", dtype=torch.int64)
        m.indices = _ptr(indices, "indices", dtype=torch.int32) if nnz else None
        m.values = _ptr(values, "values", shape=(nnz,)) if nnz else None
        m.rows, m.cols, m.nnz = rows, cols, nnz
        m.dtype = _dtype_code(values)
        return m

    def sfb_csr_check(self, indptr, indices, values, cols) -> int:
        """Number of format violations (waits for the stream)."""
        m = self._csr(indptr, indices, values, cols)
        self._grow_workspace(256)
        bad = ctypes.c_int64(0)
        self._check(lib().sfb_csr_check(self._h, ctypes.byref(m), ctypes.byref(bad)), "sfb_csr_check")
        return int(bad.value)

    def sfb_mlr_sf_csr(self, W, indptr, indices, values, y, U):
        """Enqueues U = softmax(W x_i) - onehot(y_i) for samples given as CSR rows."""
        J, D = W.shape
        m = self._csr(indptr, indices, values, D)
        B = m.rows
        need = lib().sfb_mlr_sf_csr_workspace_bytes(J, D, B, m.dtype)
        if need < 0:
            raise SfbError(int(need), "sfb_mlr_sf_csr_workspace_bytes")
        self._grow_workspace(int(need))
        if _dtype_code(U) != m.dtype:
            raise TypeError("U and the CSR values must share a dtype")
        rc = lib().sfb_mlr_sf_csr(self._h, _ptr(W, "W", dtype=torch.float32), J, D, ctypes.byref(m),
                                  _ptr(y, "y (labels)", dtype=torch.int32, shape=(B,)), _ptr(U, "U", shape=(B, J)))
        self._check(rc, "sfb_mlr_sf_csr")

    def sfb_set_csr_route(self, route: int = 0):
        """0: sfb_mlr_sf_csr picks its route per call; 1: dense product; 2: over the stored entries."""
        self._check(lib().sfb_set_csr_route(self._h, int(route)), "sfb_set_csr_route")

    def sfb_apply_csr(self, W, U, indptr, indices, values, eta, coef=None):
        """Enqueues W -= eta * sum_i coef_i u_i v_i^T with the v_i given as CSR rows (in place)."""
        J, D = W.shape
        m = self._csr(indptr, indices, values, D)
        N = m.rows
        if _dtype_code(U) != m.dtype:
            raise TypeError("U and the CSR values must share a dtype")
        need = lib().sfb_apply_csr_workspace_bytes(J, D, N, m.dtype)
        if need < 0:
            raise SfbError(int(need), "sfb_apply_csr_workspace_bytes")
        self._grow_workspace(int(need))
        rc = lib().sfb_apply_csr(self._h, _ptr(W, "W", dtype=torch.float32), J, D, _ptr(U, "U", shape=(N, J)),
                                 ctypes.byref(m),
                                 _ptr(coef, "coef", dtype=torch.float32, shape=(N,)) if coef is not None else None,
                                 float(eta))
        self._check(rc, "sfb_apply_csr")

    # -- SDCA on l2-regularised multiclass logistic regression ---------------
    def sfb_sdca_mlr_sf(self, W, X, P, lam, N, beta, dU):
        """Enqueues the dual coordinate steps of a mini-batch: dU = beta (p* - P), P += dU (in place)."""
        J, D = W.shape
        B = X.shape[0]
        need = lib().sfb_sdca_workspace_bytes(J, D, B)
        if need < 0:
            raise SfbError(int(need), "sfb_sdca_workspace_bytes")
        self._grow_workspace(int(need))
        rc = lib().sfb_sdca_mlr_sf(self._h, _ptr(W, "W", dtype=torch.float32), J, D,
                                   _ptr(X, "X", dtype=torch.float32, shape=(B, D)), B,
                                   _ptr(P, "P", dtype=torch.float32, shape=(B, J)), float(lam), int(N), float(beta),
                                   _ptr(dU, "dU", dtype=torch.float32, shape=(B, J)))
        self._check(rc, "sfb_sdca_mlr_sf")

    def sfb_dual_to_primal_l2(self, Z, W, lam):
        """Enqueues W = Z / lam."""
        J, D = W.shape
        rc = lib().sfb_dual_to_primal_l2(self._h, _ptr(Z, "Z", dtype=torch.float32, shape=(J, D)),
                                         _ptr(W, "W", dtype=torch.float32), J, D, float(lam))
        self._check(rc, "sfb_dual_to_primal_l2")

    def sfb_prox_rows(self, W, mode=SFB_PROX_PROJECT):
        J, D = W.shape
        self._check(lib().sfb_prox_rows(self._h, _ptr(W, "W", dtype=torch.float32), J, D, mode), "sfb_prox_rows")


class SspClock:
    """One sfb_ssp object (include/sfb_ssp.h): counters of BSP / SSP / ASP application of SF sets."""

    def __init__(self, P: int, s: int):
        self._h = ctypes.c_void_p()
        rc = lib().sfb_ssp_create(ctypes.byref(self._h), int(P), int(s))
        if rc != SFB_OK:
            raise SfbError(rc, "sfb_ssp_create")

    def close(self):
        if self._h:
            lib().sfb_ssp_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, v, what):
        if v < 0:
            raise SfbError(int(v), what)
        return int(v)

    def sfb_ssp_can_compute(self, p: int) -> bool:
        return bool(self._chk(lib().sfb_ssp_can_compute(self._h, int(p)), "sfb_ssp_can_compute"))

    def sfb_ssp_computed(self, p: int) -> int:
        return self._chk(lib().sfb_ssp_computed(self._h, int(p)), "sfb_ssp_computed")

    def sfb_ssp_delivered(self, p: int, q: int) -> int:
        return self._chk(lib().sfb_ssp_delivered(self._h, int(p), int(q)), "sfb_ssp_delivered")

    def sfb_ssp_pop_apply(self, p: int):
        """(q, t) of the next SF set worker p has to apply now, or None."""
        q, t = ctypes.c_int32(), ctypes.c_int64()
        rc = self._chk(lib().sfb_ssp_pop_apply(self._h, int(p), ctypes.byref(q), ctypes.byref(t)), "sfb_ssp_pop_apply")
        return (q.value, t.value) if rc else None

    def sfb_ssp_clock(self, p: int) -> int:
        return self._chk(lib().sfb_ssp_clock(self._h, int(p)), "sfb_ssp_clock")

    def sfb_ssp_tau(self, p: int, q: int) -> int:
        return self._chk(lib().sfb_ssp_tau(self._h, int(p), int(q)), "sfb_ssp_tau")

    def sfb_ssp_arrived(self, p: int, q: int) -> int:
        return self._chk(lib().sfb_ssp_arrived(self._h, int(p), int(q)), "sfb_ssp_arrived")

    def sfb_ssp_max_staleness_seen(self) -> int:
        return self._chk(lib().sfb_ssp_max_staleness_seen(self._h), "sfb_ssp_max_staleness_seen")
