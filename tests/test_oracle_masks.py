"""Pins for the mask half of the CPU oracle (no GPU).

Each test checks the oracle against something the paper or plain mathematics
fixes, computed here without the oracle's own code: exact rational arithmetic,
exhaustive subset enumeration, numpy's stable sort, hand-worked groups.
"""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
PATTERNS = [(1, 2), (2, 4), (4, 8), (1, 4), (3, 4), (2, 8)]


def _rng(seed):
    return np.random.default_rng(seed)


def _bf16_round(a):
    """Round float32 values to bf16 precision (round-to-nearest-even), keep float32."""
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def _exact_scores(w_line, f_line):
    """|w| * f as exact rationals."""
    return [abs(Fraction(float(w))) * Fraction(float(f)) for w, f in zip(w_line, f_line)]


def _brute_keep(scores, n_keep):
    """All C(m, n_keep) subsets; valid iff min(kept) >= max(pruned); lexicographically smallest."""
    m = len(scores)
    best = None
    for S in itertools.combinations(range(m), n_keep):
        rest = [b for b in range(m) if b not in S]
        if S and rest and min(scores[a] for a in S) < max(scores[b] for b in rest):
            continue
        if best is None or S < best:
            best = S
    return set(best)


def _kept(W_before, W_after):
    """Boolean kept-map; asserts kept entries are bit-identical and pruned ones are +0."""
    changed = W_before.view(np.uint32) != W_after.view(np.uint32)
    assert np.all(W_after.view(np.uint32)[changed] == 0), "pruned entries must be +0 bits"
    return ~changed


def _lines(W, axis):
    return W.T if axis == "rows" else W


# ----------------------------------------------------------------- golden --
def test_handworked_groups():
    """Groups small enough to score by hand (Sec. 3 Eq. 4 / Eq. 5 and the N:M rule)."""
    with open(os.path.join(GOLDEN, "handworked_nm.jsonl")) as fh:
        cases = [json.loads(line) for line in fh if line.strip()]
    assert len(cases) >= 7
    for c in cases:
        w = np.array([c["w"]], dtype=np.float32)
        nrm = np.array(c["norms"], dtype=np.float32)
        # as a Down-Proj row (contiguous group, norms per column) ...
        out, mask = oracle.mask_nm(w, nrm, "cols", "cols", c["alpha"], c["n_keep"], c["m"], True)
        keep = (np.array(c["keep"]) == 1)
        assert np.array_equal(out[0] != 0, keep & (w[0] != 0)), c["cite"]
        assert np.array_equal(np.unpackbits(mask[0], bitorder="little")[: c["m"]] == 1, keep), c["cite"]
        # ... and as a Gate/Up column (strided group, norms per row)
        out_t, mask_t = oracle.mask_nm(np.ascontiguousarray(w.T), nrm, "rows", "rows",
                                       c["alpha"], c["n_keep"], c["m"], True)
        assert np.array_equal(out_t[:, 0] != 0, keep & (w[0] != 0)), c["cite"]
        assert np.array_equal((mask_t[:, 0] & 1) == 1, keep), c["cite"]


# ---------------------------------------------------- P13: exact products --
def test_double_product_is_exact():
    """|w| * f in double equals the rational product for float32 and bf16 operands."""
    r = _rng(1)
    w = (r.standard_normal(4000) * 0.02).astype(np.float32)
    f = np.exp(r.standard_normal(4000) * 3).astype(np.float32)
    for ww in (w, _bf16_round(w)):
        for a, b in zip(ww, f):
            assert Fraction(abs(float(a)) * float(b)) == abs(Fraction(float(a))) * Fraction(float(b))


# ------------------------------------------------ P1 + P2: brute force ----
@pytest.mark.parametrize("n_keep,m", PATTERNS)
@pytest.mark.parametrize("axes", [("rows", "rows"), ("cols", "cols"), ("rows", "cols"), ("cols", "rows")])
@pytest.mark.parametrize("ties", [False, True])
def test_nm_matches_subset_enumeration(n_keep, m, axes, ties):
    norm_axis, group_axis = axes
    r = _rng(100 * m + n_keep + (7 if ties else 0))
    rows, cols = (3 * m, 5) if group_axis == "rows" else (5, 3 * m)
    if ties:  # few distinct magnitudes and factors => many exact ties, zeros included
        W = r.choice(np.array([-0.5, 0.0, 0.25, 0.5, 1.0], dtype=np.float32), size=(rows, cols))
        nrm = r.choice(np.array([0.0, 1.0, 4.0, 16.0], dtype=np.float32),
                       size=rows if norm_axis == "rows" else cols)
    else:
        W = (r.standard_normal((rows, cols)) * 0.02).astype(np.float32)
        nrm = np.exp(r.standard_normal(rows if norm_axis == "rows" else cols)).astype(np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    out, mask = oracle.mask_nm(W, nrm, norm_axis, group_axis, 0.5, n_keep, m, True)
    kept = _kept(W, out)
    f = np.sqrt(nrm.astype(np.float64)).astype(np.float32)  # correctly rounded float sqrt
    F = np.broadcast_to(f[:, None] if norm_axis == "rows" else f[None, :], W.shape)
    bits = np.unpackbits(mask, axis=1, bitorder="little")[:, :cols] == 1
    Wl, Fl, Kl, Bl = (_lines(a, group_axis) for a in (W, F, kept, bits))
    for line in range(Wl.shape[0]):
        for g0 in range(0, Wl.shape[1], m):
            sc = _exact_scores(Wl[line, g0:g0 + m], Fl[line, g0:g0 + m])
            want = _brute_keep(sc, n_keep)
            got_bits = {a for a in range(m) if Bl[line, g0 + a]}
            assert got_bits == want
            assert len(got_bits) == n_keep                      # P1: exact count
            # a kept zero weight is still zero in W; everything else must agree
            for a in range(m):
                if Wl[line, g0 + a] != 0:
                    assert Kl[line, g0 + a] == (a in want)


def test_nm_all_zero_and_all_equal_groups():
    """P1 on degenerate groups: the mask still has exactly n_keep ones, lowest indices."""
    for W in (np.zeros((4, 16), np.float32), np.full((4, 16), -0.5, np.float32)):
        nrm = np.ones(16, np.float32)
        for n_keep, m in PATTERNS:
            _, mask = oracle.mask_nm(W, nrm, "cols", "cols", 1.0, n_keep, m, True)
            bits = np.unpackbits(mask, axis=1, bitorder="little")[:, :16].reshape(4, 16 // m, m)
            assert np.all(bits[:, :, :n_keep] == 1) and np.all(bits[:, :, n_keep:] == 0)


def test_nm_rejects_ragged_axis():
    W = np.zeros((6, 10), np.float32)
    with pytest.raises(ValueError):
        oracle.mask_nm(W, np.ones(10, np.float32), "cols", "cols", 1.0, 2, 4)
    with pytest.raises(ValueError):
        oracle.mask_nm(W, np.ones(6, np.float32), "rows", "rows", 1.0, 2, 4)


# -------------------------------------------- P3: alpha = 0 is magnitude --
def _magnitude_keep(W, group_axis, n_keep, m):
    """Textbook magnitude N:M: stable argsort of -|w| inside every group."""
    Wl = _lines(np.abs(W.astype(np.float64)), group_axis)
    L, n = Wl.shape
    g = Wl.reshape(L, n // m, m)
    order = np.argsort(-g, axis=2, kind="stable")
    keep = np.zeros_like(g, dtype=bool)
    np.put_along_axis(keep, order[:, :, :n_keep], True, axis=2)
    keep = keep.reshape(L, n)
    return keep.T if group_axis == "rows" else keep


@pytest.mark.parametrize("n_keep,m", [(2, 4), (4, 8)])
@pytest.mark.parametrize("group_axis", ["rows", "cols"])
def test_alpha_zero_is_magnitude_pruning(n_keep, m, group_axis):
    r = _rng(3)
    W = _bf16_round(r.standard_normal((64, 48)) * 0.02)  # bf16 grid => plenty of ties
    n_norm = W.shape[0] if group_axis == "rows" else W.shape[1]
    want = _magnitude_keep(W, group_axis, n_keep, m)
    for k in range(3):
        nrm = np.exp(_rng(10 + k).standard_normal(n_norm) * 2).astype(np.float32)
        if k == 2:
            nrm[::3] = 0.0  # 0^0 = 1 by definition of the factor
        _, mask = oracle.mask_nm(W, nrm, group_axis, group_axis, 0.0, n_keep, m, True)
        bits = np.unpackbits(mask, axis=1, bitorder="little")[:, : W.shape[1]] == 1
        assert np.array_equal(bits, want)


# ----------------------------------------- P6: norms across the groups ----
@pytest.mark.parametrize("axes", [("rows", "cols"), ("cols", "rows")])
def test_constant_factor_in_group_is_magnitude_pruning(axes):
    """If the factor is the same for all members of a group the ranking is |w|'s
    (the reason Sec. 3 'Pruning Granularity' gives for input-balanced Gate/Up groups)."""
    norm_axis, group_axis = axes
    r = _rng(4)
    W = _bf16_round(r.standard_normal((32, 40)) * 0.02)
    nrm = np.exp(r.standard_normal(W.shape[0] if norm_axis == "rows" else W.shape[1])).astype(np.float32)
    _, mask = oracle.mask_nm(W, nrm, norm_axis, group_axis, 0.5, 2, 4, True)
    bits = np.unpackbits(mask, axis=1, bitorder="little")[:, : W.shape[1]] == 1
    assert np.array_equal(bits, _magnitude_keep(W, group_axis, 2, 4))


# ------------------------------------------------- P4: Down == Wanda ------
def test_down_score_is_wanda_metric():
    """Eq. 5 with norms = column norms of the layer input is Eq. 1, output-balanced."""
    r = _rng(5)
    Y = r.standard_normal((200, 64)).astype(np.float32)          # the Down-Proj input
    Wd = (r.standard_normal((24, 64)) * 0.02).astype(np.float32)
    col_norm = np.sqrt((Y.astype(np.float64) ** 2).sum(axis=0)).astype(np.float32)
    out, _ = oracle.mask_nm(Wd, col_norm, "cols", "cols", 1.0, 2, 4)
    score = [[abs(Fraction(float(Wd[i, j]))) * Fraction(float(col_norm[j])) for j in range(64)]
             for i in range(24)]
    for i in range(24):
        for g0 in range(0, 64, 4):
            order = sorted(range(4), key=lambda a: (-score[i][g0 + a], a))
            for rank, a in enumerate(order):
                assert (out[i, g0 + a] != 0) == (rank < 2)


# ------------------------------------------------ P5: scale invariance ----
def test_norm_scaling_by_powers_of_four_keeps_masks():
    r = _rng(6)
    W = (r.standard_normal((64, 32)) * 0.02).astype(np.float32)
    nrm = np.exp(r.standard_normal(64)).astype(np.float32)
    a, _ = oracle.mask_nm(W, nrm, "rows", "rows", 0.5, 2, 4)
    b, _ = oracle.mask_nm(W, nrm * np.float32(4.0), "rows", "rows", 0.5, 2, 4)   # f doubles exactly
    c, _ = oracle.mask_nm(W, nrm * np.float32(0.25), "rows", "rows", 0.5, 2, 4)
    assert np.array_equal(a, b) and np.array_equal(a, c)
    nrm_c = np.exp(r.standard_normal(32)).astype(np.float32)
    d1, _ = oracle.mask_nm(W, nrm_c, "cols", "cols", 1.0, 4, 8)
    d2, _ = oracle.mask_nm(W, nrm_c * np.float32(2.0), "cols", "cols", 1.0, 4, 8)
    assert np.array_equal(d1, d2)


# ---------------------------------------- P7: dependency coherence --------
def test_outlier_neuron_keeps_its_weights_everywhere():
    """A neuron with a huge activation norm keeps its Gate/Up row and Down column;
    with norm 0 it loses them (Fig. 1c's structural coordination)."""
    r = _rng(7)
    d, I, i_star = 16, 32, 13
    Wg = (r.uniform(0.5, 1.0, (I, d)) * r.choice([-1, 1], (I, d))).astype(np.float32)
    Wd = (r.uniform(0.5, 1.0, (d, I)) * r.choice([-1, 1], (d, I))).astype(np.float32)
    nrm = np.ones(I, np.float32)
    nrm[i_star] = 1e6
    g, _ = oracle.mask_nm(Wg, nrm, "rows", "rows", 0.5, 2, 4)
    dn, _ = oracle.mask_nm(Wd, nrm, "cols", "cols", 1.0, 2, 4)
    assert np.all(g[i_star] != 0) and np.all(dn[:, i_star] != 0)
    nrm[i_star] = 0.0
    g, _ = oracle.mask_nm(Wg, nrm, "rows", "rows", 0.5, 2, 4)
    dn, _ = oracle.mask_nm(Wd, nrm, "cols", "cols", 1.0, 2, 4)
    assert np.all(g[i_star] == 0) and np.all(dn[:, i_star] == 0)


# ------------------------------------------------- P12: idempotence -------
def test_masking_twice_changes_nothing():
    r = _rng(8)
    W = (r.standard_normal((32, 64)) * 0.02).astype(np.float32)
    nrm = np.exp(r.standard_normal(64)).astype(np.float32)
    once, _ = oracle.mask_nm(W, nrm, "cols", "cols", 1.0, 2, 4)
    twice, _ = oracle.mask_nm(once, nrm, "cols", "cols", 1.0, 2, 4)
    assert np.array_equal(once.view(np.uint32), twice.view(np.uint32))


# --------------------------------------------------- factor (Eq. 4/5) -----
def test_factor_special_cases_and_rounding():
    nrm = np.array([0.0, 1.0, 2.0, 9.0, 1e-30, 3.3e7, 0.3], dtype=np.float32)
    assert np.array_equal(oracle.factor(nrm, 0.0), np.ones(7, np.float32))
    assert np.array_equal(oracle.factor(nrm, 1.0), nrm)
    half = oracle.factor(nrm, 0.5)
    assert half[0] == 0.0 and half[1] == 1.0 and half[3] == 3.0
    for x, s in zip(nrm, half):  # correctly rounded: s is the float nearest sqrt(x), checked exactly
        s_dn, s_up = np.nextafter(s, np.float32(0)), np.nextafter(s, np.float32(np.inf))
        lo = (Fraction(float(s)) + Fraction(float(s_dn))) / 2
        hi = (Fraction(float(s)) + Fraction(float(s_up))) / 2
        assert lo * lo <= Fraction(float(x)) <= hi * hi
    quarter = oracle.factor(np.array([16.0, 81.0], np.float32), 0.25)
    assert np.array_equal(quarter, np.array([2.0, 3.0], np.float32))


# ------------------------------------------------------ unstructured ------
@pytest.mark.parametrize("axes", [("rows", "rows"), ("cols", "cols"), ("cols", "rows")])
@pytest.mark.parametrize("ties", [False, True])
def test_unstructured_matches_exact_sort(axes, ties):
    norm_axis, group_axis = axes
    r = _rng(20 + ties)
    rows, cols = 37, 19
    if ties:
        W = r.choice(np.array([-0.5, 0.0, 0.25, 0.5], dtype=np.float32), size=(rows, cols))
        nrm = r.choice(np.array([0.0, 1.0, 4.0], dtype=np.float32), size=rows if norm_axis == "rows" else cols)
    else:
        W = (r.standard_normal((rows, cols)) * 0.02).astype(np.float32)
        nrm = np.exp(r.standard_normal(rows if norm_axis == "rows" else cols)).astype(np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    f = np.sqrt(nrm.astype(np.float64)).astype(np.float32)
    F = np.broadcast_to(f[:, None] if norm_axis == "rows" else f[None, :], W.shape)
    length = rows if group_axis == "rows" else cols
    for n_prune in (0, 1, length // 2, length - 1, length):
        out, mask = oracle.mask_unstructured(W, nrm, norm_axis, group_axis, 0.5, n_prune, True)
        bits = np.unpackbits(mask, axis=1, bitorder="little")[:, :cols] == 1
        kept = _kept(W, out)
        Wl, Fl, Bl, Kl = (_lines(a, group_axis) for a in (W, F, bits, kept))
        for line in range(Wl.shape[0]):
            sc = _exact_scores(Wl[line], Fl[line])
            order = sorted(range(length), key=lambda a: (-sc[a], a))
            want = set(order[: length - n_prune])
            assert {a for a in range(length) if Bl[line, a]} == want
            assert Bl[line].sum() == length - n_prune
            for a in range(length):
                if Wl[line, a] != 0:
                    assert Kl[line, a] == (a in want)


def test_unstructured_equals_nm_when_line_is_one_group():
    """A line of length m with n_prune = m - n_keep is a single N:M group."""
    r = _rng(30)
    W = (r.standard_normal((16, 8)) * 0.02).astype(np.float32)
    nrm = np.exp(r.standard_normal(8)).astype(np.float32)
    a, _ = oracle.mask_nm(W, nrm, "cols", "cols", 1.0, 4, 8)
    b, _ = oracle.mask_unstructured(W, nrm, "cols", "cols", 1.0, 4)
    assert np.array_equal(a, b)


def test_unstructured_rejects_bad_quota():
    W = np.zeros((4, 8), np.float32)
    for bad in (-1, 9):
        with pytest.raises(ValueError):
            oracle.mask_unstructured(W, np.ones(8, np.float32), "cols", "cols", 1.0, bad)
