"""Pins for the MLP output (Eq. 2 then Eq. 3) and the 2:4 compressed form in the CPU oracle (no GPU).

Closed forms, a library matrix product, the identity that ties the MLP output to the pinned
squared sums, a hand-worked example and the round trip; no expected value comes from the
function under test.
"""
import json
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "handworked_compress_24.jsonl")


# ------------------------------------------------------------------ Eq. 3 --
def test_one_hot_weights_closed_form():
    """X has a constant-1 column c; Wg_i = gamma_i e_c makes the gate a constant, Wu_i = beta_i e_{j_i}
    makes the up projection one input feature: y_i = silu(gamma_i) beta_i X[t, j_i], and the output
    is that vector times Wd^T."""
    rng = np.random.default_rng(1)
    T, d, I = 9, 6, 5
    X = rng.standard_normal((T, d)).astype(np.float32)
    c = 2
    X[:, c] = 1.0
    gamma = np.array([0.0, 1.0, -2.0, 0.5, 3.0])
    beta = np.array([1.0, -0.5, 2.0, 4.0, 0.25])
    pick = np.array([0, 1, 3, 4, 5])
    Wg = np.zeros((I, d), dtype=np.float32)
    Wu = np.zeros((I, d), dtype=np.float32)
    Wg[np.arange(I), c] = gamma
    Wu[np.arange(I), pick] = beta
    Wd = rng.standard_normal((d, I)).astype(np.float32)
    silu = gamma / (1.0 + np.exp(-gamma))
    y = silu[None, :] * beta[None, :] * X[:, pick].astype(np.float64)
    want = y @ Wd.astype(np.float64).T
    got = oracle.mlp_forward(X, Wg, Wu, Wd, "silu")
    assert got.shape == (T, d)
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=1e-15)


def test_relu_with_positive_gate_is_a_library_product():
    """ReLU of a positive gate is the identity: out = ((X Wg^T) * (X Wu^T)) Wd^T by numpy in float64."""
    rng = np.random.default_rng(2)
    T, d, I = 7, 5, 11
    X = np.abs(rng.standard_normal((T, d))).astype(np.float32)
    Wg = np.abs(rng.standard_normal((I, d))).astype(np.float32)
    Wu = rng.standard_normal((I, d)).astype(np.float32)
    Wd = rng.standard_normal((d, I)).astype(np.float32)
    X64, Wg64, Wu64, Wd64 = (a.astype(np.float64) for a in (X, Wg, Wu, Wd))
    y = (X64 @ Wg64.T) * (X64 @ Wu64.T)
    got, ab = oracle.mlp_forward(X, Wg, Wu, Wd, "relu", want_abs=True)
    np.testing.assert_allclose(got, y @ Wd64.T, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ab, np.abs(y) @ np.abs(Wd64).T, rtol=1e-12, atol=1e-13)
    # a negative gate gives nothing at all
    assert np.all(oracle.mlp_forward(X, -Wg, Wu, Wd, "relu") == 0.0)


def test_selecting_down_projection_reproduces_the_pinned_squared_sums():
    """Wd = rows of the identity picks single neurons: out[t, j] = y[t, i_j], so the column sums of
    out^2 are the squared norms that the (separately pinned) stage-1 oracle returns."""
    rng = np.random.default_rng(3)
    T, d, I = 40, 4, 10
    X = rng.standard_normal((T, d)).astype(np.float32)
    Wg = rng.standard_normal((I, d)).astype(np.float32)
    Wu = rng.standard_normal((I, d)).astype(np.float32)
    sel = np.array([7, 0, 3, 9])
    Wd = np.zeros((d, I), dtype=np.float32)
    Wd[np.arange(d), sel] = 1.0
    for kind in ("silu", "gelu_tanh", "gelu_erf", "relu"):
        out = oracle.mlp_forward(X, Wg, Wu, Wd, kind)
        np.testing.assert_allclose((out ** 2).sum(0), oracle.sumsq(X, Wg, Wu, kind, neurons=sel), rtol=1e-13)


def test_token_selection_and_operand_roles():
    rng = np.random.default_rng(4)
    T, d, I = 12, 3, 8
    X = rng.standard_normal((T, d)).astype(np.float32)
    Wg = rng.standard_normal((I, d)).astype(np.float32)
    Wu = rng.standard_normal((I, d)).astype(np.float32)
    Wd = rng.standard_normal((d, I)).astype(np.float32)
    full = oracle.mlp_forward(X, Wg, Wu, Wd, "silu")
    tok = np.array([11, 0, 5])
    assert np.array_equal(oracle.mlp_forward(X, Wg, Wu, Wd, "silu", tokens=tok), full[tok])
    # gate and up are not interchangeable, and Wd is used as [d, d_int] (not transposed)
    assert not np.allclose(oracle.mlp_forward(X, Wu, Wg, Wd, "silu"), full)
    one = np.zeros_like(Wd)
    one[1, 6] = 2.0   # output feature 1 reads neuron 6 only
    y6 = oracle.mlp_forward(X, Wg, Wu, one, "silu")
    g = X.astype(np.float64) @ Wg[6].astype(np.float64)
    u = X.astype(np.float64) @ Wu[6].astype(np.float64)
    np.testing.assert_allclose(y6[:, 1], 2.0 * g / (1.0 + np.exp(-g)) * u, rtol=1e-13)
    assert np.all(y6[:, [0, 2]] == 0.0)


# ------------------------------------------------------------- 2:4 form --
def _decompress(values, meta, group_axis, shape):
    """The inverse map, written from the format's definition (plain loops)."""
    rows, cols = shape
    W = np.zeros(shape, dtype=np.float32)
    if group_axis == "cols":
        for r in range(rows):
            for g in range(cols // 4):
                code = (meta[r, g // 2] >> (4 * (g & 1))) & 15
                W[r, 4 * g + (code & 3)] = values[r, 2 * g]
                W[r, 4 * g + (code >> 2)] = values[r, 2 * g + 1]
    else:
        for c in range(cols):
            for g in range(rows // 4):
                code = (meta[g, c // 2] >> (4 * (c & 1))) & 15
                W[4 * g + (code & 3), c] = values[2 * g, c]
                W[4 * g + (code >> 2), c] = values[2 * g + 1, c]
    return W


def test_hand_worked_examples():
    with open(GOLDEN) as f:
        cases = [json.loads(line) for line in f if line.strip()]
    assert len(cases) >= 3
    for case in cases:
        W = np.array(case["W"], dtype=np.float32)
        values, meta, surplus = oracle.compress_24(W, case["group_axis"])
        assert values.tolist() == case["values"], case["why"]
        assert meta.tolist() == case["meta"], case["why"]
        assert surplus == case["surplus"]


@pytest.mark.parametrize("group_axis", ["cols", "rows"])
def test_round_trip_and_code_invariants(group_axis):
    rng = np.random.default_rng(5)
    rows, cols = 24, 40
    W = rng.standard_normal((rows, cols)).astype(np.float32)
    # make it 2:4 along the axis with random kept pairs; a tenth of the kept weights are zero too
    lines = W if group_axis == "cols" else W.T
    for line in lines:
        for g in range(line.size // 4):
            drop = rng.choice(4, size=2, replace=False)
            line[4 * g + drop] = 0.0
    W[rng.random(W.shape) < 0.1] = 0.0
    values, meta, surplus = oracle.compress_24(W, group_axis)
    assert surplus == 0
    assert values.shape == ((rows, cols // 2) if group_axis == "cols" else (rows // 2, cols))
    assert np.array_equal(_decompress(values, meta, group_axis, W.shape), W)
    lo, hi = meta & 15, meta >> 4
    for code in (lo, hi):
        assert np.all((code & 3) < (code >> 2))          # p0 < p1 in every nibble
    # half of the elements are stored, none invented
    assert np.count_nonzero(values) == np.count_nonzero(W)


def test_dense_groups_are_counted_and_bad_shapes_rejected():
    W = np.ones((4, 8), dtype=np.float32)
    assert oracle.compress_24(W, "cols")[2] == 8 and oracle.compress_24(W, "rows")[2] == 8
    with pytest.raises(ValueError):
        oracle.compress_24(np.ones((4, 12), dtype=np.float32), "cols")   # cols % 8
    with pytest.raises(ValueError):
        oracle.compress_24(np.ones((6, 8), dtype=np.float32), "rows")    # rows % 4


# ------------------------------------------------- Eq. 3 from the 2:4 form --
def test_down_sparse24_hand_worked_row():
    """One output feature, two groups: values (2, -3 | 0.5, 4) at positions (1, 3 | 0, 2):
    out = 2 y1 - 3 y3 + 0.5 y4 + 4 y6, written out by hand for y = 1..8."""
    values = np.array([[2.0, -3.0, 0.5, 4.0]], dtype=np.float32)
    meta = np.array([[(1 | 3 << 2) | (0 | 2 << 2) << 4]], dtype=np.uint8)
    Y = np.arange(1, 9, dtype=np.float32)[None, :]
    out, ab = oracle.down_sparse24(Y, values, meta, want_abs=True)
    assert out.tolist() == [[2 * 2 - 3 * 4 + 0.5 * 5 + 4 * 7]]        # y1 = 2, y3 = 4, y4 = 5, y6 = 7
    assert ab.tolist() == [[4 + 12 + 2.5 + 28]]


def test_down_sparse24_equals_a_library_product_with_the_decoded_matrix():
    rng = np.random.default_rng(8)
    d, d_int, T = 12, 64, 9
    W = rng.standard_normal((d, d_int)).astype(np.float32)
    for row in W:
        for g in range(d_int // 4):
            row[4 * g + rng.choice(4, size=2, replace=False)] = 0.0
    W[rng.random(W.shape) < 0.1] = 0.0
    values, meta, surplus = oracle.compress_24(W, "cols")
    assert surplus == 0 and np.array_equal(_decompress(values, meta, "cols", W.shape), W)
    Y = rng.standard_normal((T, d_int)).astype(np.float32)
    want = Y.astype(np.float64) @ W.astype(np.float64).T
    got = oracle.down_sparse24(Y, values, meta)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-14)
    tok = np.array([8, 0, 3])
    assert np.array_equal(oracle.down_sparse24(Y, values, meta, tokens=tok), got[tok])
    # and it continues Eq. 2: with y from the dense oracle the two routes to the block output agree
    X = rng.standard_normal((T, d)).astype(np.float32)
    Wg = rng.standard_normal((d_int, d)).astype(np.float32)
    Wu = rng.standard_normal((d_int, d)).astype(np.float32)
    full = oracle.mlp_forward(X, Wg, Wu, W, "silu")
    g64 = X.astype(np.float64) @ Wg.astype(np.float64).T
    y = (g64 / (1.0 + np.exp(-g64)) * (X.astype(np.float64) @ Wu.astype(np.float64).T)).astype(np.float32)
    np.testing.assert_allclose(oracle.down_sparse24(y, values, meta), full, rtol=1e-5, atol=1e-6)
