"""The parity metrics themselves (CPU): mistakes planted in the oracle's output must fail them.

The MLR first factor holds one entry near -1 per row and J - 1 probabilities of order 1/J; a metric whose
scale is set by the label entry passes probabilities that are wrong by a large factor.  mlr_u_check must not.
"""
import numpy as np
import pytest

import sfb_synth as S
from parity import TOL_BF16, TOL_F32, mlr_u_check, rel_err


def _case(oracle, J, D, B, seed):
    W = S.normal_matrix(J, D, 0.05, seed=seed)
    X, y = S.mlr_batch(J, D, B, seed=seed, zero_frac=0.5, bf16=True)
    U, _ = oracle.mlr_sf(W, X, y)
    return U, y


@pytest.mark.parametrize("J", [2048, 40000])
def test_mlr_u_check_catches_what_the_plain_metric_misses(oracle, J):
    U, y = _case(oracle, J, 16, 6, seed=3)
    B = U.shape[0]
    idx = np.arange(B)
    bf = S.round_to_bf16(U.astype(np.float32)).astype(np.float64)
    # honest bf16 rounding of the oracle's result passes
    mlr_u_check(bf, U, y, TOL_BF16)
    mlr_u_check(U.astype(np.float32), U, y, TOL_F32)
    # (a) every probability doubled
    bad = U.copy()
    lab = bad[idx, y].copy()
    bad *= 2.0
    bad[idx, y] = lab
    if J >= 40000:
        assert rel_err(bad, U) <= TOL_BF16          # the plain metric is blind to it at this row length
    with pytest.raises(AssertionError):
        mlr_u_check(bad, U, y, TOL_BF16)
    # (b) one tile of 256 classes off by 50 %
    bad = U.copy()
    bad[:, 512:768] *= 1.5
    bad[idx, y] = U[idx, y]
    with pytest.raises(AssertionError):
        mlr_u_check(bad, U, y, TOL_BF16)
    # (c) a wrong normaliser of one row (1.5 %): element-wise within bf16's tolerance, caught by the row factor
    bad = bf.copy()
    bad[2] *= 1.015
    bad[2, y[2]] = bf[2, y[2]]
    with pytest.raises(AssertionError):
        mlr_u_check(bad, U, y, TOL_BF16)
    # (d) the label entry without its -1
    bad = bf.copy()
    bad[1, y[1]] += 1.0
    with pytest.raises(AssertionError):
        mlr_u_check(bad, U, y, TOL_BF16)
    # (e) a single probability replaced by its neighbour's class (index slip inside a row)
    bad = U.copy()
    j = (y[0] + 7) % J
    bad[0, j] = U[0, j] * 3.0
    with pytest.raises(AssertionError):
        mlr_u_check(bad, U, y, TOL_BF16)


def test_dml_follow_kink_only_touches_pairs_at_the_kink(oracle):
    """Hand-built pairs: one dissimilar pair a hair below the margin, one clearly active, one clearly inactive.
    Whatever the library decided for the first, the oracle's row follows it; a wrong decision on the others
    stays a mismatch."""
    from parity import dml_follow_kink
    K = D = 4
    W = np.eye(K, D)
    X = np.zeros((3, D)); Y = np.zeros((3, D))
    X[0, 0] = np.sqrt(1.0 - 2e-6)      # d = 1 - 2e-6
    X[1, 1] = 0.5                      # d = 0.25
    X[2, 2] = 2.0                      # d = 4
    sim = np.array([-1, -1, -1], dtype=np.int8)
    Uo, _, no = oracle.dml_sf(W, X, Y, sim, margin=1.0)
    assert no == 2 and np.any(Uo[0] != 0)
    # the library took the other side for pair 0, and (wrongly) switched pair 2 on
    got = Uo.copy()
    got[0] = 0.0
    got[2] = -2.0 * X[2]
    U2, n2, near = dml_follow_kink(oracle, Uo.copy(), no, got, W, X, Y, sim, 1.0, 1e-5)
    assert near == 1 and n2 == 1
    np.testing.assert_array_equal(U2[0], 0.0)
    np.testing.assert_array_equal(U2[1], Uo[1])
    np.testing.assert_array_equal(U2[2], 0.0)          # not at the kink: the oracle's own decision stands
    assert rel_err(got, U2) > TOL_F32
    # and back: the library active where the oracle (at d = 1 + 2e-6) is not
    X[0, 0] = np.sqrt(1.0 + 2e-6)
    Uo, _, no = oracle.dml_sf(W, X, Y, sim, margin=1.0)
    assert no == 1 and not np.any(Uo[0] != 0)
    got = Uo.copy()
    got[0] = -2.0 * X[0]
    U2, n2, near = dml_follow_kink(oracle, Uo.copy(), no, got, W, X, Y, sim, 1.0, 1e-5)
    assert near == 1 and n2 == 2
    np.testing.assert_allclose(U2[0], -2.0 * X[0], rtol=1e-15)
