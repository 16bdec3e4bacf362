"""ctypes loader for the CPU oracle (``sfb_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Importable from ``tests/``, from
``__graft_entry__.smoke()`` and from ``bench.py``'s cpu_baseline leg; the product
package never imports this module and this module never imports the product.

All wrappers take NumPy arrays, convert them (exactly) to contiguous fp64 and
return fp64 results.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sfb_oracle.c")
_LIB = os.path.join(_HERE, "libsfb_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        i64 = ctypes.c_int64
        lib.sfbo_num_threads.restype = ctypes.c_int
        lib.sfbo_apply.argtypes = [dp, dp, dp, i64, i64, i64, ctypes.c_double]
        lib.sfbo_apply.restype = None
        lib.sfbo_apply_signed.argtypes = [dp, dp, dp, dp, i64, i64, i64, ctypes.c_double]
        lib.sfbo_apply_signed.restype = None
        lib.sfbo_mlr_sf.argtypes = [dp, dp, ctypes.POINTER(ctypes.c_int32), i64, i64, i64, dp, dp]
        lib.sfbo_mlr_sf.restype = None
        ip64 = ctypes.POINTER(ctypes.c_int64)
        ip32 = ctypes.POINTER(ctypes.c_int32)
        lib.sfbo_mlr_sf_csr.argtypes = [dp, ip64, ip32, dp, ip32, i64, i64, i64, dp, dp]
        lib.sfbo_mlr_sf_csr.restype = None
        lib.sfbo_apply_csr.argtypes = [dp, dp, ip64, ip32, dp, i64, i64, i64, ctypes.c_double]
        lib.sfbo_apply_csr.restype = None
        lib.sfbo_dml_sf.argtypes = [dp, dp, dp, ctypes.POINTER(ctypes.c_int8), i64, i64, i64,
                                    ctypes.c_double, dp, dp, ctypes.POINTER(ctypes.c_int32), dp]
        lib.sfbo_dml_sf.restype = None
        lib.sfbo_sc_lipschitz.argtypes = [dp, i64, i64, ctypes.c_int32]
        lib.sfbo_sc_lipschitz.restype = ctypes.c_double
        lib.sfbo_sc_sf.argtypes = [dp, dp, i64, i64, i64, ctypes.c_double, ctypes.c_int32,
                                   ctypes.c_double, dp, dp]
        lib.sfbo_sc_sf.restype = None
        lib.sfbo_prox_rows.argtypes = [dp, i64, i64, ctypes.c_int32]
        lib.sfbo_prox_rows.restype = None
        _lib = lib
    return _lib


def _f64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and a.shape != tuple(shape):
        raise ValueError("expected shape %r, got %r" % (tuple(shape), a.shape))
    return a


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads() -> int:
    return int(_load().sfbo_num_threads())


PROX_PROJECT = 0
PROX_NORMALIZE = 1


def apply(W, U, V, eta):
    """Returns W - eta * sum_i u_i v_i^T (new fp64 array)."""
    W = np.array(W, dtype=np.float64, order="C", copy=True)
    J, D = W.shape
    U = _f64(U)
    V = _f64(V)
    N = U.shape[0]
    if U.shape != (N, J) or V.shape != (N, D):
        raise ValueError("U must be [N][J] and V [N][D]")
    _load().sfbo_apply(_dp(W), _dp(U), _dp(V), N, J, D, float(eta))
    return W


def apply_signed(W, U, V, coef, eta):
    """Returns W - eta * sum_i coef_i u_i v_i^T (new fp64 array)."""
    W = np.array(W, dtype=np.float64, order="C", copy=True)
    J, D = W.shape
    U = _f64(U)
    V = _f64(V)
    c = _f64(coef)
    N = U.shape[0]
    if U.shape != (N, J) or V.shape != (N, D) or c.shape != (N,):
        raise ValueError("U must be [N][J], V [N][D], coef [N]")
    _load().sfbo_apply_signed(_dp(W), _dp(U), _dp(V), _dp(c), N, J, D, float(eta))
    return W


def mlr_sf(W, X, y, with_loss=False):
    """MLR sufficient factors.  Returns (U [B][J], V [B][D]) (V is X)."""
    W = _f64(W)
    X = _f64(X)
    J, D = W.shape
    B = X.shape[0]
    if X.shape != (B, D):
        raise ValueError("X must be [B][D]")
    y = np.ascontiguousarray(y, dtype=np.int32)
    if y.shape != (B,) or (B and (y.min() < 0 or y.max() >= J)):
        raise ValueError("labels must be [B] in [0, J)")
    U = np.empty((B, J), dtype=np.float64)
    loss = np.empty((B,), dtype=np.float64)
    _load().sfbo_mlr_sf(_dp(W), _dp(X), y.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                        J, D, B, _dp(U), _dp(loss))
    if with_loss:
        return U, X, loss
    return U, X


def _csr(indptr, indices, values, rows, cols):
    """Validated CSR triple: int64 indptr [rows+1], int32 indices and fp64 values [nnz];
    column indices distinct and in range within every row."""
    indptr = np.ascontiguousarray(indptr, dtype=np.int64)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    values = _f64(values)
    if indptr.shape != (rows + 1,) or indptr[0] != 0 or np.any(np.diff(indptr) < 0):
        raise ValueError("indptr must be [rows+1], start at 0 and not decrease")
    nnz = int(indptr[-1])
    if indices.shape != (nnz,) or values.shape != (nnz,):
        raise ValueError("indices and values must have indptr[-1] entries")
    if nnz and (indices.min() < 0 or indices.max() >= cols):
        raise ValueError("column index out of range")
    for i in range(rows):
        seg = indices[indptr[i]:indptr[i + 1]]
        if np.unique(seg).size != seg.size:
            raise ValueError("duplicate column index in row %d" % i)
    return indptr, indices, values


def mlr_sf_csr(W, indptr, indices, values, y, with_loss=False):
    """MLR first factors U [B][J] for samples given as CSR rows (non-zeros only)."""
    W = _f64(W)
    J, D = W.shape
    B = len(indptr) - 1
    indptr, indices, values = _csr(indptr, indices, values, B, D)
    y = np.ascontiguousarray(y, dtype=np.int32)
    if y.shape != (B,) or (B and (y.min() < 0 or y.max() >= J)):
        raise ValueError("labels must be [B] in [0, J)")
    U = np.empty((B, J), dtype=np.float64)
    loss = np.empty((B,), dtype=np.float64)
    i32p = ctypes.POINTER(ctypes.c_int32)
    _load().sfbo_mlr_sf_csr(_dp(W), indptr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                            indices.ctypes.data_as(i32p), _dp(values), y.ctypes.data_as(i32p),
                            J, D, B, _dp(U), _dp(loss))
    return (U, loss) if with_loss else U


def apply_csr(W, U, indptr, indices, values, eta):
    """Returns W - eta * sum_i u_i v_i^T with the v_i given as CSR rows (new fp64 array)."""
    W = np.array(W, dtype=np.float64, order="C", copy=True)
    J, D = W.shape
    U = _f64(U)
    N = U.shape[0]
    if U.shape != (N, J):
        raise ValueError("U must be [N][J]")
    indptr, indices, values = _csr(indptr, indices, values, N, D)
    _load().sfbo_apply_csr(_dp(W), _dp(U), indptr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                           indices.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _dp(values),
                           N, J, D, float(eta))
    return W


def dml_sf(W, X, Y, sim, margin=1.0, with_loss=False):
    """DML sufficient factors.  Returns (U [B][K], V [B][D], n_active)."""
    W = _f64(W)
    X = _f64(X)
    Y = _f64(Y)
    K, D = W.shape
    B = X.shape[0]
    if X.shape != (B, D) or Y.shape != (B, D):
        raise ValueError("X, Y must be [B][D]")
    sim = np.ascontiguousarray(sim, dtype=np.int8)
    if sim.shape != (B,):
        raise ValueError("sim must be [B]")
    U = np.empty((B, K), dtype=np.float64)
    V = np.empty((B, D), dtype=np.float64)
    loss = np.empty((B,), dtype=np.float64)
    n_active = ctypes.c_int32(0)
    _load().sfbo_dml_sf(_dp(W), _dp(X), _dp(Y), sim.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)),
                        K, D, B, float(margin), _dp(U), _dp(V), ctypes.byref(n_active), _dp(loss))
    if with_loss:
        return U, V, int(n_active.value), loss
    return U, V, int(n_active.value)


def sc_lipschitz(W, power_iters=10):
    W = _f64(W)
    J, D = W.shape
    return float(_load().sfbo_sc_lipschitz(_dp(W), J, D, int(power_iters)))


def sc_sf(W, X, lam=0.1, ista_iters=20, power_iters=10, L=None):
    """Sparse-coding sufficient factors.  Returns (U = codes [B][J], V = residuals [B][D], L)."""
    W = _f64(W)
    X = _f64(X)
    J, D = W.shape
    B = X.shape[0]
    if X.shape != (B, D):
        raise ValueError("X must be [B][D]")
    if L is None:
        L = sc_lipschitz(W, power_iters)
    U = np.empty((B, J), dtype=np.float64)
    V = np.empty((B, D), dtype=np.float64)
    _load().sfbo_sc_sf(_dp(W), _dp(X), J, D, B, float(lam), int(ista_iters), float(L), _dp(U), _dp(V))
    return U, V, float(L)


def prox_rows(W, mode=PROX_PROJECT):
    W = np.array(W, dtype=np.float64, order="C", copy=True)
    J, D = W.shape
    _load().sfbo_prox_rows(_dp(W), J, D, int(mode))
    return W
