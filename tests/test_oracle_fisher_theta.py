"""Pins for the oracle's pair-level importance (Eq. 8) and cumulative-threshold removal rule (Alg. 1)
against closed forms, element-by-element loops, brute force over subsets and the already pinned
top-k selection (no GPU, no product code)."""
import itertools

import numpy as np
import pytest

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import synth


# ---- Eq. 8 ------------------------------------------------------------------------------
def test_fisher_constant_gradients_closed_form():
    """Every entry of both gradients equal to c: each member's mean square is c^2, so I = c^2 / |D|
    whatever the shapes - the 1/|W_k| factors make the two members weigh the same."""
    for kind, g1s, g2s, groups, n in ((O.PAIR_QK, (12, 5), (12, 9), 3, 4), (O.PAIR_VO, (12, 5), (7, 12), 3, 4),
                                      (O.PAIR_FFN, (10, 3), (6, 10), 1, 10)):
        got = O.pair_fisher(kind, np.full(g1s, 0.5), np.full(g2s, 0.5), groups, n, 8.0)
        np.testing.assert_allclose(got, np.full(groups, 0.25 / 8.0), rtol=1e-14)
    got = O.pair_fisher(O.PAIR_FFN_GATED, np.full((10, 3), 2.0), np.full((6, 10), 2.0), 1, 10, 4.0, g1b=np.full((10, 3), 2.0))
    np.testing.assert_allclose(got, [1.0], rtol=1e-14)


def test_fisher_matches_element_loops():
    """Independent restatement with scalar loops over the entries each head owns."""
    h, n, d1, d2, D = 3, 4, 5, 6, 17.0
    g1 = synth.normal(3, 1, (h * n, d1)).astype(np.float64)
    gk = synth.normal(3, 2, (h * n, d2)).astype(np.float64)      # QK: rows of the second member
    go = synth.normal(3, 3, (d2, h * n)).astype(np.float64)      # VO: columns of the second member
    for kind, g2 in ((O.PAIR_QK, gk), (O.PAIR_VO, go)):
        want = []
        for g in range(h):
            s1 = sum(g1[g * n + j, c] ** 2 for j in range(n) for c in range(d1)) / (n * d1)
            if kind == O.PAIR_QK:
                s2 = sum(g2[g * n + j, c] ** 2 for j in range(n) for c in range(d2)) / (n * d2)
            else:
                s2 = sum(g2[r, g * n + j] ** 2 for j in range(n) for r in range(d2)) / (n * d2)
            want.append(0.5 * (s1 + s2) / D)
        np.testing.assert_allclose(O.pair_fisher(kind, g1, g2, h, n, D), want, rtol=1e-13)


def test_fisher_members_balanced_and_layout_consistent():
    h, n, d = 2, 6, 5
    g1 = synth.normal(4, 1, (h * n, d)).astype(np.float64)
    g2 = synth.normal(4, 2, (h * n, 3 * d)).astype(np.float64)
    base = O.pair_fisher(O.PAIR_QK, g1, g2, h, n, 1.0)
    # the second member stored transposed (columns aligned) is the same pair
    np.testing.assert_allclose(O.pair_fisher(O.PAIR_VO, g1, np.ascontiguousarray(g2.T), h, n, 1.0), base, rtol=1e-14)
    # scaling one member by a changes only that member's half: I' - I = (a^2 - 1)/2 * mean(g1^2)
    a = 3.0
    m1 = np.array([(g1[g * n:(g + 1) * n] ** 2).mean() for g in range(h)])
    np.testing.assert_allclose(O.pair_fisher(O.PAIR_QK, a * g1, g2, h, n, 1.0) - base, 0.5 * (a * a - 1) * m1, rtol=1e-12)
    # repeating the second member's entries (more parameters, same mean square) changes nothing
    np.testing.assert_allclose(O.pair_fisher(O.PAIR_QK, g1, np.concatenate([g2, g2], axis=1), h, n, 1.0), base, rtol=1e-14)
    # |D| divides, heads permute
    np.testing.assert_allclose(O.pair_fisher(O.PAIR_QK, g1, g2, h, n, 5.0), base / 5.0, rtol=1e-14)
    perm = np.concatenate([np.arange(n, 2 * n), np.arange(0, n)])
    np.testing.assert_allclose(O.pair_fisher(O.PAIR_QK, g1[perm], g2[perm], h, n, 1.0), base[::-1], rtol=1e-14)


def test_fisher_gated_first_member_is_both_matrices():
    n, d = 8, 4
    gg, gu = synth.normal(5, 1, (n, d)).astype(np.float64), synth.normal(5, 2, (n, d)).astype(np.float64)
    gd = synth.normal(5, 3, (d, n)).astype(np.float64)
    want = 0.5 * (((gg ** 2).sum() + (gu ** 2).sum()) / (2 * n * d) + (gd ** 2).mean()) / 3.0
    np.testing.assert_allclose(O.pair_fisher(O.PAIR_FFN_GATED, gg, gd, 1, n, 3.0, g1b=gu), [want], rtol=1e-14)


# ---- Alg. 1 removal loop -------------------------------------------------------------------
def _mass(row):
    return [int(v) for v in O.theta_mass(row)]


def test_theta_mass_is_exact_and_clipped():
    s = np.array([0.0, -0.0, 1.0, 0.5, 2.0, -3.0, np.nan, 2.0 ** -32, 3 * 2.0 ** -33, 0.75 + 2.0 ** -24], dtype=np.float32)
    assert _mass(s) == [0, 0, 2 ** 32, 2 ** 31, 2 ** 32, 0, 0, 1, 1, 3 * 2 ** 30 + 2 ** 8]


@pytest.mark.parametrize("seed", range(6))
def test_theta_rule_equals_smallest_sufficient_topk(seed):
    """The kept set is the top-k* of the (separately pinned) top-k selection, k* the smallest k >= 1 whose
    mass reaches the bound: removing ascending until the next removal would fall below the bound is the
    same as keeping the smallest sufficient head of the descending order."""
    rng = np.random.default_rng(seed)
    n = 23
    s = rng.random((4, n)).astype(np.float32)
    s[1, rng.integers(0, n, 6)] = s[1, 3]            # ties
    s[2, :5] = 0.0
    s[3, 2] = np.nan
    s /= np.float32(np.nansum(s, axis=1, keepdims=True).max())
    for theta in (0.3, 0.5, 0.9, 0.99):
        idx, ks = O.select_theta(s, theta)
        for g in range(4):
            q = _mass(s[g])
            bound = int(np.ceil(np.float64(np.float32(theta)) * np.float64(sum(q))))
            kstar = next(k for k in range(1, n + 1) if sum(q[i] for i in O.select_topk(s[g:g + 1], k)[0]) >= bound)
            assert ks[g] == kstar
            assert np.array_equal(idx[g, :kstar], O.select_topk(s[g:g + 1], kstar)[0])
            assert np.all(idx[g, kstar:] == -1)


def test_theta_rule_brute_force_over_subsets():
    """Tiny groups without ties: among all subsets whose mass reaches the bound, the rule keeps the one with
    the fewest units - and for that size the one with the largest mass (unique without ties)."""
    rng = np.random.default_rng(11)
    for trial in range(20):
        n = int(rng.integers(2, 8))
        s = rng.permutation(np.arange(1, n + 1)).astype(np.float32) / np.float32(n * (n + 1) / 2 * 1.5)
        theta = float(rng.choice([0.2, 0.45, 0.7, 0.95]))
        q = _mass(s)
        bound = int(np.ceil(np.float64(np.float32(theta)) * np.float64(sum(q))))
        best = None
        for k in range(1, n + 1):
            ok = [c for c in itertools.combinations(range(n), k) if sum(q[i] for i in c) >= bound]
            if ok:
                best = max(ok, key=lambda c: sum(q[i] for i in c))
                break
        idx, ks = O.select_theta(s[None, :], theta)
        assert ks[0] == len(best) and tuple(idx[0, :ks[0]]) == best


def test_theta_rule_limits_monotonicity_and_ties():
    s = np.array([[0.125, 0.25, 0.25, 0.125, 0.0, 0.25]], dtype=np.float32)
    idx, ks = O.select_theta(s, 1.0)           # only massless units can go
    assert ks[0] == 5 and list(idx[0, :5]) == [0, 1, 2, 3, 5]
    idx, ks = O.select_theta(s, 0.0)           # one unit always stays: the largest, lowest index on ties
    assert ks[0] == 1 and idx[0, 0] == 1
    idx, ks = O.select_theta(s, 0.75)          # 0.125 (index 3, then 0) removed: kept mass exactly 0.75
    assert list(idx[0, :ks[0]]) == [1, 2, 5]
    idx, ks = O.select_theta(s, 0.8)           # only one of the two 0.125 units can go: the higher index
    assert list(idx[0, :ks[0]]) == [0, 1, 2, 5]
    rng = np.random.default_rng(5)
    r = rng.random((1, 64)).astype(np.float32) / np.float32(40)
    prev = 0
    for theta in (0.1, 0.3, 0.5, 0.7, 0.9, 0.99, 1.0):
        k = int(O.select_theta(r, theta)[1][0])
        assert k >= prev
        prev = k
    # halving every score (exact in binary) halves every mass: same kept set
    a = O.select_theta(r, 0.6)
    b = O.select_theta(r * np.float32(0.5), 0.6)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
