"""Host-side checks of the seeded input generators."""
import numpy as np

import sfb_synth as S


def test_round_to_bf16_ties_to_even_and_bits():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 0.0, 1.0 + 2 ** -9], dtype=np.float32)
    r = S.round_to_bf16(x)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    np.testing.assert_array_equal(r, np.array([1.0, 1.0, 1.0 + 2 ** -6, -2.5, 0.0, 1.0], dtype=np.float32))
    b = S.bf16_bits(r)
    assert b.dtype == np.int16
    np.testing.assert_array_equal((b.view(np.uint16).astype(np.uint32) << 16).view(np.float32), r)


def test_generators_are_seeded_and_shaped():
    X1, y1 = S.mlr_batch(10, 16, 8, seed=3, step=2, zero_frac=0.9, bf16=True)
    X2, y2 = S.mlr_batch(10, 16, 8, seed=3, step=2, zero_frac=0.9, bf16=True)
    np.testing.assert_array_equal(X1, X2); np.testing.assert_array_equal(y1, y2)
    X3, _ = S.mlr_batch(10, 16, 8, seed=3, step=3, zero_frac=0.9, bf16=True)
    assert not np.array_equal(X1, X3)
    assert X1.dtype == np.float32 and y1.dtype == np.int32 and y1.min() >= 0 and y1.max() < 10
    U, V = S.mlr_peer_sf(12, 6, 5, seed=0, step=1, peer=4)
    assert U.shape == (5, 12) and V.shape == (5, 6)
    np.testing.assert_allclose(U.sum(axis=1), 0.0, atol=1e-6)
    X, Y, sim = S.dml_batch(8, 6, seed=0)
    assert list(sim) == [1, 1, 1, -1, -1, -1] and X.shape == Y.shape == (6, 8)
    W = S.sc_dictionary(7, 9, seed=0)
    np.testing.assert_allclose(np.linalg.norm(W, axis=1), 1.0, atol=1e-6)


def test_zero_fraction():
    X, _ = S.mlr_batch(4, 1000, 64, seed=1, zero_frac=0.9)
    frac = np.mean(X == 0.0)
    assert 0.88 < frac < 0.92
