"""Pins for the input-feature norms of Eq. 1 (the Wanda metric) in the CPU oracle (no GPU).

Closed forms and a hand-worked selection; none of the expected values comes from the oracle.
"""
import numpy as np
import pytest

import oracle


def test_sum_of_squares_of_integers_closed_form():
    """Column j holds (j + 1) * (1, 2, ..., T): sum = (j + 1)^2 T (T + 1) (2T + 1) / 6, exact in double."""
    T, d = 300, 7
    X = (np.arange(1, T + 1, dtype=np.float32)[:, None] * np.arange(1, d + 1, dtype=np.float32)[None, :])
    got = oracle.input_sumsq(X)
    want = np.array([(j + 1) ** 2 * T * (T + 1) * (2 * T + 1) // 6 for j in range(d)], dtype=np.float64)
    assert np.array_equal(got, want)


def test_columns_are_independent_and_signs_do_not_matter():
    T = 64
    X = np.zeros((T, 3), dtype=np.float32)
    X[:, 0] = 0.5 * (-1.0) ** np.arange(T)      # alternating +-0.5: T / 4
    X[5, 1] = -3.0                              # one entry: 9
    got = oracle.input_sumsq(X)                 # column 2 stays empty: 0
    assert got.tolist() == [T / 4, 9.0, 0.0]
    X[:, 2] = 100.0
    assert oracle.input_sumsq(X)[:2].tolist() == [T / 4, 9.0]


def test_axis_is_tokens_not_features():
    """A non-square X with a different constant in every column: d results of T c^2 each
    (a transposed read would give T results or mix the constants)."""
    T, d = 5, 11
    c = np.arange(1, d + 1, dtype=np.float32)
    got = oracle.input_sumsq(np.tile(c, (T, 1)))
    assert got.shape == (d,) and np.array_equal(got, T * c.astype(np.float64) ** 2)


def test_chunks_accumulate_and_leading_dimension():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((96, 40)).astype(np.float32)
    whole = oracle.input_sumsq(X)
    acc = oracle.input_sumsq(X[:50])
    oracle.input_sumsq(X[50:], out=acc)
    assert np.allclose(acc, whole, rtol=1e-15)
    wide = np.full((96, 56), 7.0, dtype=np.float32)
    wide[:, :40] = X
    assert np.array_equal(oracle.input_sumsq(wide[:, :40]), whole)


def test_equals_the_library_sum_of_squares():
    rng = np.random.default_rng(4)
    X = (rng.standard_normal((257, 33)) * rng.uniform(0.01, 30, 33)).astype(np.float32)
    want = np.einsum("tj,tj->j", X.astype(np.float64), X.astype(np.float64))
    assert np.allclose(oracle.input_sumsq(X), want, rtol=1e-14)
    assert np.allclose(oracle.norms(oracle.input_sumsq(X)), np.linalg.norm(X.astype(np.float64), axis=0), rtol=1e-14)


def test_hand_worked_wanda_selection():
    """Eq. 1 end to end on numbers small enough to do by hand.  Two tokens x = (3, 0, 1, 2) and
    (4, 0, 1, 0): norms (5, 0, sqrt 2, 2).  One output row w = (1, 9, -3, 2): scores
    (5, 0, 4.24.., 4); per output, 2:4 keeps the scores 5 and 4.24 -> positions 0 and 2."""
    X = np.array([[3, 0, 1, 2], [4, 0, 1, 0]], dtype=np.float32)
    nrm = oracle.norms(oracle.input_sumsq(X)).astype(np.float32)
    assert nrm.tolist() == pytest.approx([5.0, 0.0, 2 ** 0.5, 2.0], rel=1e-7)
    W = np.array([[1, 9, -3, 2]], dtype=np.float32)
    pruned, mask = oracle.mask_nm(W, nrm, "cols", "cols", 1.0, 2, 4, want_mask=True)
    assert pruned.tolist() == [[1.0, 0.0, -3.0, 0.0]]
    assert mask.tolist() == [[0b0101]]
