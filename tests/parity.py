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


def mlr_u_check(got, ref, y, tol, factor_tol=None, label_tol=None):
    """Checks MLR first factors U = softmax - onehot (rows of `got` against the oracle's `ref`, labels `y`).

    A row holds one entry near -1 (the label) and J - 1 probabilities of order 1/J.  Taken over the whole row,
    rms(r) is the label entry's (about 1/sqrt(J)), and rel_err would pass probabilities that are wrong by a
    large factor.  So the label entry is compared on its own, the element-wise metric is taken with the label
    entries masked out (its rms is then the probabilities' own), and the least-squares factor between the two
    rows (label aside) must be 1: rounding errors average out over a row, a wrong normaliser or a wrong tile
    does not.  Returns the masked element-wise error.
    """
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    B = r.shape[0]
    if r.size == 0:
        return 0.0
    if factor_tol is None:
        # bf16 path: half the element-wise tolerance.  The weighted mean of a row's relative errors does not
        # average out when a few large probabilities carry the row (each is off by the error of its own
        # logit, |dz| of several 1e-3 with bf16 parameters and logits of a few units) or when all entries are
        # alike (an all-zero sample: every probability is 1/J and rounds the same way, up to 2^-8).  Callers
        # with small logits and spread rows pass a tighter bound.  fp32: a tenth of the element-wise tolerance.
        factor_tol = 0.5 * tol if tol >= 1e-3 else 0.1 * tol
    idx = np.arange(B)
    y = np.asarray(y)
    lab = np.abs(g[idx, y] - r[idx, y])
    # the label entry is p - 1: spacing 2^-8 near -1 in bf16, 2^-24 in fp32
    assert np.all(lab <= (label_tol if label_tol is not None else max(tol, 1e-6))), float(lab.max())
    gm = g.copy()
    rm = r.copy()
    gm[idx, y] = 0.0
    rm[idx, y] = 0.0
    n = max(r.size - B, 1)
    rms = np.sqrt(np.sum(rm * rm) / n)
    den = np.abs(rm) + rms
    den[den == 0.0] = 1.0
    err = float(np.max(np.abs(gm - rm) / den))
    assert err <= tol, (err, tol)
    den_f = np.sum(rm * rm, axis=1)
    ok = den_f > 0
    factor = np.sum(gm * rm, axis=1)[ok] / den_f[ok]
    assert np.all(np.abs(factor - 1.0) < factor_tol), (float(factor.min()), float(factor.max()))
    return err


def dml_follow_kink(oracle, Uo, n_active, U_got, W, X, Y, sim, margin, width):
    """A dissimilar pair whose squared distance is within `width` of the margin may fall on either side of the
    hinge's kink in fp32: both decisions are valid.  For those pairs the oracle's row follows the decision the
    library took (its active row, from an oracle call with the margin moved out of the way, or zero), so that
    everything else stays comparable element by element.  Returns (Uo, n_active, number of such pairs)."""
    d = np.sum(((np.asarray(X, dtype=np.float64) - Y) @ np.asarray(W, dtype=np.float64).T) ** 2, axis=1)
    near = np.flatnonzero((np.asarray(sim) < 0) & (np.abs(d - margin) < width))
    if near.size:
        U_on, _, _ = oracle.dml_sf(W, X, Y, sim, margin=margin + 2.0 * width + 1.0)
        for i in near:
            took = bool(np.any(U_got[i] != 0))
            n_active += int(took) - int(np.any(Uo[i] != 0))
            Uo[i] = U_on[i] if took else 0.0
    return Uo, n_active, int(near.size)
