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
