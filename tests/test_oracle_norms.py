"""Pins for the norm half of the CPU oracle (no GPU).

Closed forms, hand-computable cases and invariants that fix Eq. 2 followed by
the squared sum over tokens, none of them computed with the oracle's own code.
"""
import math

import numpy as np
import pytest

import oracle

ACTS = ["silu", "gelu_tanh", "gelu_erf", "relu"]


def _rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------- sigma spots --
def test_activation_spot_values():
    for kind in ACTS:
        assert oracle.act(0.0, kind) == 0.0
    assert oracle.act(-1.0, "relu") == 0.0 and oracle.act(2.5, "relu") == 2.5
    # Swish(1) = logistic(1); written through tanh so it is not the oracle's expression
    assert oracle.act(1.0, "silu") == pytest.approx(0.5 * (1.0 + math.tanh(0.5)), rel=1e-15)
    assert oracle.act(1.0, "silu") == pytest.approx(0.7310585786300049, rel=1e-15)
    # GeLU(1) = Phi(1), the standard normal CDF at one standard deviation
    assert oracle.act(1.0, "gelu_erf") == pytest.approx(0.8413447460685429, rel=1e-14)
    assert oracle.act(-1.0, "gelu_erf") == pytest.approx(-(1 - 0.8413447460685429), rel=1e-13)
    # tanh form, via the logistic identity 0.5 (1 + tanh z) = 1 / (1 + e^{-2z})
    z = math.sqrt(2 / math.pi) * (1.0 + 0.044715)
    assert oracle.act(1.0, "gelu_tanh") == pytest.approx(1.0 / (1.0 + math.exp(-2 * z)), rel=1e-14)
    assert abs(oracle.act(1.0, "gelu_tanh") - oracle.act(1.0, "gelu_erf")) < 5e-4
    # antisymmetry relations: silu(g) - silu(-g) = g, gelu(g) - gelu(-g) = g
    for kind in ("silu", "gelu_tanh", "gelu_erf"):
        for g in (0.3, 2.0, 7.5):
            assert oracle.act(g, kind) - oracle.act(-g, kind) == pytest.approx(g, rel=1e-13)
    # far tails
    assert oracle.act(-800.0, "silu") == 0.0 and oracle.act(800.0, "silu") == 800.0
    assert oracle.act(40.0, "gelu_tanh") == 40.0


# ------------------------------------------------------ hand-worked 2x2 ---
def test_reglu_two_tokens_by_hand():
    X = np.array([[1, 2], [-3, 4]], dtype=np.float32)
    Wu = np.array([[2, 0.5]], dtype=np.float32)
    # gate = [-1, -7] -> ReLU kills both tokens
    assert oracle.sumsq(X, np.array([[1, -1]], np.float32), Wu, "relu")[0] == 0.0
    # gate = [1, 7], up = [3, -4] -> y = [3, -28] -> 9 + 784
    assert oracle.sumsq(X, np.array([[-1, 1]], np.float32), Wu, "relu")[0] == 793.0
    assert oracle.norms([793.0])[0] == pytest.approx(math.sqrt(793.0), rel=1e-15)


def test_gate_and_up_are_not_interchangeable():
    """sigma acts on the first projection only (Eq. 2): swapping Wg and Wu changes y."""
    X = np.array([[1.0, 0.0], [0.0, 1.0]], dtype=np.float32)
    A = np.array([[2.0, -1.0]], np.float32)
    B = np.array([[0.5, 3.0]], np.float32)
    silu = lambda g: g / (1 + math.exp(-g))
    want_ab = (silu(2.0) * 0.5) ** 2 + (silu(-1.0) * 3.0) ** 2
    want_ba = (silu(0.5) * 2.0) ** 2 + (silu(3.0) * -1.0) ** 2
    assert oracle.sumsq(X, A, B, "silu")[0] == pytest.approx(want_ab, rel=1e-14)
    assert oracle.sumsq(X, B, A, "silu")[0] == pytest.approx(want_ba, rel=1e-14)
    assert abs(want_ab - want_ba) > 1.0


# ------------------------------------------------ P8 / P9: closed forms ---
@pytest.mark.parametrize("kind", ACTS)
def test_constant_gate_gives_gram_quadratic_form(kind):
    """With gate == gamma on every token, sumsq_i = sigma(gamma)^2 * wu^T (X^T X) wu."""
    r = _rng(11)
    T, d, I, c = 300, 24, 10, 5
    X = r.standard_normal((T, d)).astype(np.float32)
    X[:, c] = 1.0
    gammas = np.linspace(-2.0, 3.0, I).astype(np.float32)
    Wg = np.zeros((I, d), np.float32)
    Wg[:, c] = gammas
    Wu = (r.standard_normal((I, d)) * 0.1).astype(np.float32)
    got = oracle.sumsq(X, Wg, Wu, kind)
    X64, Wu64 = X.astype(np.float64), Wu.astype(np.float64)
    gram = X64.T @ X64
    sig = {"silu": lambda g: g * 0.5 * (1 + math.tanh(g / 2)),
           "gelu_tanh": lambda g: g / (1 + math.exp(-2 * math.sqrt(2 / math.pi) * (g + 0.044715 * g ** 3))),
           "gelu_erf": lambda g: g * 0.5 * math.erfc(-g / math.sqrt(2)),
           "relu": lambda g: max(g, 0.0)}[kind]
    want = np.array([sig(float(gammas[i])) ** 2 * (Wu64[i] @ gram @ Wu64[i]) for i in range(I)])
    assert np.allclose(got, want, rtol=1e-11, atol=1e-300)


def test_single_channel_up_reduces_to_input_feature_norm():
    """Additionally Wu_i = beta e_j  =>  norm_i = |sigma(gamma) beta| * ||X[:, j]||_2 (Eq. 1's norm)."""
    r = _rng(12)
    T, d, c, j = 500, 16, 3, 9
    X = r.standard_normal((T, d)).astype(np.float32)
    X[:, c] = 1.0
    Wg = np.zeros((2, d), np.float32); Wg[:, c] = [1.5, -0.75]
    Wu = np.zeros((2, d), np.float32); Wu[:, j] = [2.0, -4.0]
    got = oracle.norms(oracle.sumsq(X, Wg, Wu, "silu"))
    colnorm = math.sqrt(float((X[:, j].astype(np.float64) ** 2).sum()))
    silu = lambda g: g / (1 + math.exp(-g))
    want = [abs(silu(1.5) * 2.0) * colnorm, abs(silu(-0.75) * -4.0) * colnorm]
    assert np.allclose(got, want, rtol=1e-12)


# --------------------------------------- independent dense recomputation --
@pytest.mark.parametrize("kind", ACTS)
def test_against_blas_recomputation(kind):
    """Same definition through a float64 BLAS matmul and scipy special functions."""
    from scipy import special

    r = _rng(13)
    T, d, I = 257, 96, 41
    X = r.standard_normal((T, d)).astype(np.float32)
    X[:, 7] *= 20
    Wg = (r.standard_normal((I, d)) * 0.05).astype(np.float32)
    Wu = (r.standard_normal((I, d)) * 0.05).astype(np.float32)
    G = X.astype(np.float64) @ Wg.astype(np.float64).T
    U = X.astype(np.float64) @ Wu.astype(np.float64).T
    s = {"silu": G * special.expit(G),
         "gelu_tanh": G * special.expit(2 * np.sqrt(2 / np.pi) * (G + 0.044715 * G ** 3)),
         "gelu_erf": G * special.ndtr(G),
         "relu": np.maximum(G, 0)}[kind]
    want = ((s * U) ** 2).sum(axis=0)
    assert np.allclose(oracle.sumsq(X, Wg, Wu, kind), want, rtol=1e-11)


# ----------------------------------- P11: chunks, permutations, subsets ---
def test_chunk_additivity_token_permutation_and_neuron_subset():
    r = _rng(14)
    T, d, I = 200, 32, 12
    X = r.standard_normal((T, d)).astype(np.float32)
    Wg = (r.standard_normal((I, d)) * 0.1).astype(np.float32)
    Wu = (r.standard_normal((I, d)) * 0.1).astype(np.float32)
    whole = oracle.sumsq(X, Wg, Wu, "silu")
    acc = None
    for lo, hi in ((0, 64), (64, 65), (65, 200)):
        acc = oracle.sumsq(np.ascontiguousarray(X[lo:hi]), Wg, Wu, "silu", out=acc)
    assert np.allclose(acc, whole, rtol=1e-13)
    perm = r.permutation(T)
    assert np.allclose(oracle.sumsq(np.ascontiguousarray(X[perm]), Wg, Wu, "silu"), whole, rtol=1e-13)
    sel = np.array([11, 0, 5])
    assert np.array_equal(oracle.sumsq(X, Wg, Wu, "silu", neurons=sel), whole[sel])
    # strided views (leading dimension larger than the logical width) read the same numbers
    Xp = np.zeros((T, d + 8), np.float32); Xp[:, :d] = X
    Wgp = np.zeros((I, d + 4), np.float32); Wgp[:, :d] = Wg
    Wup = np.zeros((I, d + 4), np.float32); Wup[:, :d] = Wu
    assert np.array_equal(oracle.sumsq(Xp[:, :d], Wgp[:, :d], Wup[:, :d], "silu"), whole)


def test_scaling_laws():
    """sumsq is quadratic in Wu; for ReLU it is also quadratic in a positive gate scale."""
    r = _rng(15)
    X = r.standard_normal((64, 16)).astype(np.float32)
    Wg = (r.standard_normal((5, 16)) * 0.1).astype(np.float32)
    Wu = (r.standard_normal((5, 16)) * 0.1).astype(np.float32)
    base = oracle.sumsq(X, Wg, Wu, "silu")
    assert np.allclose(oracle.sumsq(X, Wg, Wu * np.float32(-2), "silu"), 4 * base, rtol=1e-14)
    rl = oracle.sumsq(X, Wg, Wu, "relu")
    assert np.allclose(oracle.sumsq(X, Wg * np.float32(4), Wu, "relu"), 16 * rl, rtol=1e-14)
