"""Error metrics used by the parity tests (test-side only)."""
import numpy as np

TOL_F32 = 1e-4     # fp32 paths: max relative error
TOL_BF16 = 2e-2    # bf16 inputs, fp32 accumulate


def rel_err(got, ref):
    """max_ij |g - r| / (|r| + rms(r)).

    Element-wise relative error with the tensor's rms added to the denominator,
    so that entries which are tiny only through cancellation do not ask for
    more digits than any finite-precision sum can deliver.
    """
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    if r.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(r * r))
    den = np.abs(r) + rms
    den[den == 0.0] = 1.0
    return float(np.max(np.abs(g - r) / den))


def max_rel(got, ref):
    """max|g - r| / max|r| (reported alongside rel_err)."""
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    m = np.max(np.abs(r)) if r.size else 0.0
    return float(np.max(np.abs(g - r)) / (m if m > 0 else 1.0)) if r.size else 0.0


def trajectory_check(Wg, Wref, W0, steps, tol):
    """After `steps` updates from W0: max |g - r| within tol times the rms distance moved, plus the fp32
    rounding of the stored values themselves."""
    Wref = np.asarray(Wref)
    moved = Wref - W0
    bound = tol * np.sqrt(np.mean(moved * moved)) + 2 * steps * np.spacing(np.float32(np.max(np.abs(Wref))))
    err = np.max(np.abs(Wg.astype(np.float64) - Wref))
    assert err <= bound, (err, bound)
